// Batches of sequences of different lengths (the method keeps the full KV cache of every
// sequence and says nothing about unequal lengths; Algorithm 2's Full branch streams all of a
// sequence's rows): the deal of the self-scheduling Full kernel's workgroups to the (batch,
// KV head) pairs in proportion to their rows, made on the device from the device-resident
// lengths right before the streaming kernel.  With the same number of workgroups for every
// pair, the longest sequences would set the kernel time while the compute units of the short
// ones idle.
#include "device_util.h"
#include "launch.h"

namespace hylra {

// Sum over the workgroup of one value per thread (every thread gets it).
DEVI long long plan_block_sum(long long v, long long* s_red) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) v += __shfl_xor(v, m, 64);
    __syncthreads();                              // s_red may still be read from the previous call
    if (lane == 0) s_red[wave] = v;
    __syncthreads();
    return s_red[0] + s_red[1] + s_red[2] + s_red[3];
}

// One workgroup.  Every KV head has the slots g * S * B .. (g + 1) * S * B - 1 of the launch;
// within them sequence b owns n_b consecutive ones from its exclusive prefix sum on.  n_b =
// max(1, ceil(T_b / L)) with T_b the sequence's wave tiles and L the smallest load (tiles per
// workgroup) for which the batch needs no more than S * B workgroups: no deal has a smaller
// largest load, and it is never above the even deal's ceil(max T / S).
__global__ __launch_bounds__(256) void ragged_plan_kernel(RaggedPlanParams p) {
    __shared__ int s_t[kMaxRaggedBatch];         // tiles per sequence
    __shared__ int s_n[kMaxRaggedBatch];         // workgroups per sequence, then their inclusive prefix sums
    __shared__ long long s_red[4];
    __shared__ int s_wave[4];
    __shared__ int s_carry;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    long long sum = 0;
    for (int b = tid; b < p.B; b += 256) {
        const int rows = seq_rows(p.seq_lens, b, p.N);
        const int t = (rows + p.tile - 1) / p.tile;
        s_t[b] = t;
        sum += t;
    }
    const long long total = plan_block_sum(sum, s_red);
    const long long budget = (long long)p.S * p.B;
    // smallest L in [lo, hi] whose demand fits the budget; hi = ceil(max T / S) always fits
    // (every sequence then needs at most S workgroups), and so does any larger L
    int lo = (int)max(1LL, (total + budget - 1) / budget);
    int hi = max(lo, (p.N / p.tile + p.S) / p.S + 1);
    while (lo < hi) {
        const int mid = lo + (hi - lo) / 2;
        long long need = 0;
        for (int b = tid; b < p.B; b += 256) need += max(1, (s_t[b] + mid - 1) / mid);
        if (plan_block_sum(need, s_red) <= budget) hi = mid;
        else lo = mid + 1;
    }
    const int L = lo;
    for (int b = tid; b < p.B; b += 256) s_n[b] = max(1, (s_t[b] + L - 1) / L);
    if (tid == 0) s_carry = 0;
    __syncthreads();

    // inclusive prefix sums, 256 sequences at a time
    for (int b0 = 0; b0 < p.B; b0 += 256) {
        const int b = b0 + tid;
        int incl = b < p.B ? s_n[b] : 0;
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) {
            const int up = __shfl_up(incl, m, 64);
            if (lane >= m) incl += up;
        }
        if (lane == 63) s_wave[wave] = incl;
        __syncthreads();
        int before = s_carry;
        for (int w = 0; w < wave; ++w) before += s_wave[w];
        if (b < p.B) s_n[b] = before + incl;
        __syncthreads();
        if (tid == 255) s_carry = before + incl;
        __syncthreads();
    }

    // the pairs' entries
    const int per_head = p.S * p.B;
    for (int b = tid; b < p.B; b += 256) {
        const int end = s_n[b], begin = b ? s_n[b - 1] : 0;
        for (int g = 0; g < p.Hkv; ++g) p.pair_map[(int64_t)b * p.Hkv + g] = make_int2(g * per_head + begin, end - begin);
    }
    // the workgroups' entries: slot j of a head belongs to the first sequence whose prefix sum exceeds j
    const int used = s_n[p.B - 1];
    for (int j = tid; j < per_head; j += 256) {
        int seq = 0, w = 0, n = 0, begin = 0, rows = 0;
        if (j < used) {
            int a = 0, z = p.B - 1;                         // smallest b with s_n[b] > j
            while (a < z) {
                const int mid = (a + z) >> 1;
                if (s_n[mid] > j) z = mid;
                else a = mid + 1;
            }
            seq = a;
            begin = a ? s_n[a - 1] : 0;
            w = j - begin;
            n = s_n[a] - begin;
            rows = seq_rows(p.seq_lens, a, p.N);
        }
        for (int g = 0; g < p.Hkv; ++g) {
            // (slot = workgroup of the grid.  Spreading a pair's slots over the two halves of the grid, as
            // the kernels do for equal lengths, measured 2 % slower at batch 8 and no faster at batch 32.)
            const int x = g * per_head + j;
            p.wg_map[x] = make_int4(seq * p.Hkv + g, w | (n << 16), g * per_head + begin, rows);
        }
    }
}

hipError_t launch_ragged_plan(const RaggedPlanParams& p, hipStream_t st) {
    // (a sequence's workgroups, at most S * B, must fit the upper half of a map entry's second word)
    if (p.B < 1 || p.B > kMaxRaggedBatch || p.S < 1 || (int64_t)p.S * p.B > kMaxRaggedWgs || p.tile < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL(ragged_plan_kernel, dim3(1), dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace hylra
