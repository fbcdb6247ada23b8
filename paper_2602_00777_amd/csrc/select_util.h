// Workgroup-level scan helpers and constants shared by the top-k selection kernels
// (1024 threads = 16 wave64 per workgroup).
#pragma once
#include "device_util.h"

namespace hylra {

constexpr int SEL_THREADS = 1024;
constexpr int SEL_WAVES = SEL_THREADS / 64;
constexpr int SEL_BINS = 4096;
constexpr int SEL_CAP = 1024;
constexpr int SEL_ML_CAP = 2048;   // (max, sum) pairs of one KV head's partials staged in LDS

DEVI int wave_incl_scan(int v, int lane) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int n = __shfl_up(v, d, 64);
        if (lane >= d) v += n;
    }
    return v;
}

// Exclusive prefix over the workgroup in thread order; total receives the sum.
// s_wave holds SEL_WAVES + 1 ints.  Contains barriers: every thread must call it.
DEVI int block_excl_scan(int v, int* s_wave, int& total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int incl = wave_incl_scan(v, lane);
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        const int w = lane < SEL_WAVES ? s_wave[lane] : 0;
        const int wi = wave_incl_scan(w, lane);
        if (lane < SEL_WAVES) s_wave[lane] = wi - w;
        if (lane == SEL_WAVES - 1) s_wave[SEL_WAVES] = wi;
    }
    __syncthreads();
    const int base = s_wave[wave];
    total = s_wave[SEL_WAVES];
    __syncthreads();
    return base + incl - v;
}

// Inclusive prefix sum over the 64 lanes of a wave with DPP only (row_shr 1/2/4/8 inside
// each 16-lane row, then row_bcast15 / row_bcast31 carry the row totals forward).
DEVI int wave_incl_scan_dpp(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);
    return v;
}

// E independent exclusive prefix sums at once.  Value j of thread t precedes value j' of
// thread t' iff (j, t) < (j', t') lexicographically -- the row order of the register-resident
// scores.  s_tot holds E * SEL_WAVES + 1 ints.  Returns the grand total.  Contains barriers:
// every thread must call it.
template <int E>
DEVI int multi_scan(const int (&cnt)[E], int (&base)[E], int* s_tot) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl[E];
#pragma unroll
    for (int j = 0; j < E; ++j) {
        incl[j] = wave_incl_scan_dpp(cnt[j]);
        if (lane == 63) s_tot[j * SEL_WAVES + wave] = incl[j];
    }
    __syncthreads();
    if (wave == 0) {
        constexpr int PER = (E * SEL_WAVES + 63) / 64;
        int a[PER], sum = 0;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int q = lane * PER + u;
            a[u] = q < E * SEL_WAVES ? s_tot[q] : 0;
            sum += a[u];
        }
        int run = wave_incl_scan_dpp(sum) - sum;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int q = lane * PER + u;
            if (q < E * SEL_WAVES) s_tot[q] = run;
            run += a[u];
        }
        if (lane == 63) s_tot[E * SEL_WAVES] = run;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < E; ++j) base[j] = s_tot[j * SEL_WAVES + wave] + incl[j] - cnt[j];
    const int total = s_tot[E * SEL_WAVES];
    __syncthreads();
    return total;
}

DEVI int score_bin(float x, float lo, float inv_w) {
    const int b = (int)((x - lo) * inv_w);
    return min(max(b, 0), SEL_BINS - 1);
}

}  // namespace hylra
