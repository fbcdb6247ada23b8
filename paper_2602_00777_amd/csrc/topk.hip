// Full layer, after the streaming pass: merge of the split partials into the attention
// output (Algorithm 2, "O <- Softmax(S) V") and the EXACT selection of the k positions with
// the largest group-mean score (Algorithm 2, "I <- TopK(S, B)"; ties to the lower position,
// ascending order).  One launch, C workgroups of 1024 threads per (batch, KV head).
//
// Rows are ranked by (key descending, position ascending), key = the order-preserving 32-bit
// image of the fp32 score.  The selection is a radix select on the key, 12 + 12 + 8 bits:
//   level 1  a histogram of the top 12 key bits over all of the pair's rows.  It is COMPLETE
//            when this kernel starts: the streaming kernel bins the scores it has staged in
//            LDS and adds its non-empty bins to the pair's histogram in memory (for the
//            kernels that do not, score_hist_kernel below does it in a launch of its own).
//            Every workgroup reads it and finds the bin T1 that holds the k-th best row.
//   level 2  the rows of bin T1 (a few per cent of all rows) are binned on the next 12 bits
//            in LDS, by every workgroup for itself; bin T2 holds the k-th best row.
//   level 3  the rows whose top 24 bits equal (T1, T2) -- a handful unless scores tie -- are
//            ranked pairwise in LDS; if they do not fit there (massive ties), one more
//            histogram over the last 8 bits settles the threshold key and the rows equal to it
//            are taken in position order.
// Workgroup c of a pair emits the selected rows of chunk c (4096 * E_OWN consecutive rows, kept
// in registers) at the place in the output that the selected rows of the chunks before it
// leave; for that it counts those rows itself.  No workgroup waits for another one.  Rows
// outside the own chunk are kept in registers too when the pair's rows fit there (E_ALL > 0,
// up to 65536 rows), else they are re-read (from the L2 / memory-side cache) in each pass.
// The histogram in memory is zeroed again by the workgroup of the pair that read it last (an
// arrival counter), so the next Full layer finds it empty.
#include "launch.h"
#include "select_util.h"

namespace hylra {

constexpr int kTopkFineBins = 4096;

// Threshold bin of a histogram whose bins NB-1-4t .. NB-4-4t sit in h4[0..3] of thread t: the
// bin T that holds the k-th largest row and the number of rows in the bins above it.  s_pick
// must hold (SEL_BINS, 0) on entry (what comes back when k = 0).  Contains barriers.
DEVI void threshold_pick(const int (&h4)[4], int k, int* s_wave, int* s_pick, int& T, int& above) {
    const int tid = threadIdx.x;
    const int local = h4[0] + h4[1] + h4[2] + h4[3];
    int total;
    const int excl = block_excl_scan(local, s_wave, total);
    if (excl < k && k <= excl + local) {
        int c = excl;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (c < k && k <= c + h4[e]) {
                s_pick[0] = SEL_BINS - 1 - (4 * tid + e);
                s_pick[1] = c;
            }
            c += h4[e];
        }
    }
    __syncthreads();
    T = s_pick[0];
    above = s_pick[1];
    __syncthreads();                 // s_pick may be written again
}

DEVI float f4_at(const float4& v, int e) { return e == 0 ? v.x : e == 1 ? v.y : e == 2 ? v.z : v.w; }

template <int E_OWN, int E_ALL>
__global__ __launch_bounds__(SEL_THREADS) void topk_kernel(TopkParams p) {
    constexpr bool ALLREG = E_ALL > 0;
    constexpr int NREG = ALLREG ? E_ALL : E_OWN;
    static_assert(!ALLREG || E_ALL % E_OWN == 0, "chunks tile the register-resident rows");
    static_assert(E_OWN <= 16, "selection masks hold 4 * E_OWN bits");
    __shared__ int s_hist[kTopkFineBins];
    __shared__ uint32_t s_ckey[SEL_CAP];
    __shared__ int s_cpos[SEL_CAP];
    __shared__ unsigned long long s_sel[SEL_THREADS];   // candidates of this chunk that made the cut
    __shared__ int s_wave[SEL_WAVES + 1];
    __shared__ int s_tot[E_OWN * SEL_WAVES + 1];
    __shared__ int s_pick[2];
    __shared__ int s_cand, s_before, s_before_eq, s_kr, s_last;
    __shared__ uint32_t s_tau;

    const int c = blockIdx.x, g = blockIdx.y, b = blockIdx.z, C = gridDim.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int64_t pair = (int64_t)b * p.Hkv + g;
    const PartView pv = part_view(p.pair_map, pair, p.n_splits);
    const int S = pv.S, D = p.D, G = p.G;
    const int64_t hb = pv.first * G;              // first partial of the pair's first head

    // this sequence ranks its first N rows (none: merge only) and selects k of them
    const int N = p.idx ? seq_units(p.seq_lens, b, p.N, p.sel_block) : 0, k = min(p.k, N);
    const int n4 = (N + 3) >> 2;
    const float* __restrict__ sc = p.scores + pair * p.score_stride;
    const float4* __restrict__ sc4 = reinterpret_cast<const float4*>(sc);
    int32_t* __restrict__ dst = p.idx + pair * (int64_t)p.k;
    const int first4 = c * E_OWN * SEL_THREADS;                   // the chunk's first float4 group
    const int chunk_pos0 = 4 * first4, chunk_pos1 = chunk_pos0 + 4 * E_OWN * SEL_THREADS;
    if (p.idx && c == 0)
        for (int i = k + tid; i < p.k; i += SEL_THREADS) dst[i] = -1;  // entries beyond a short sequence

    // ---- loads first: the rows (the own chunk in registers 0 .. E_OWN - 1) and the histogram ----
    // register j holds float4 group grp(j) of the pair
    auto grp = [&](int j) {
        return ALLREG ? ((j + c * E_OWN) & (E_ALL - 1)) * SEL_THREADS + tid : first4 + j * SEL_THREADS + tid;
    };
    float4 v[NREG];
#pragma unroll
    for (int j = 0; j < NREG; ++j) {
        const int i = grp(j);
        v[j] = i < n4 ? sc4[i] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    int h4[4] = {0, 0, 0, 0};
    int* __restrict__ gh = p.ghist + pair * SEL_BINS;
    if (p.idx) {
        const int4 h = *reinterpret_cast<const int4*>(gh + SEL_BINS - 4 - 4 * tid);
        h4[0] = h.w, h4[1] = h.z, h4[2] = h.y, h4[3] = h.x;
    }
    for (int i = tid; i < kTopkFineBins; i += SEL_THREADS) s_hist[i] = 0;
    s_sel[tid] = 0;
    if (tid == 0) s_cand = 0, s_before = 0, s_before_eq = 0, s_last = 0, s_pick[0] = SEL_BINS, s_pick[1] = 0;

    // ---- attention output: this workgroup's share of the G*D outputs of the KV head.  16 lanes
    // per output element, each merging every 16th partial. ----
    {
        constexpr int L = 16;
        const int share = (G * D + C - 1) / C;
        const int64_t head0 = (int64_t)b * p.Hq + (int64_t)g * G;
        const int sub = tid & (L - 1), sgrp = tid / L;
        const int end = min(G * D, (c + 1) * share);
        for (int i = c * share + sgrp; i < end; i += SEL_THREADS / L) {
            const int h = i / D, col = i - h * D;
            const float* ml = p.part_ml + (hb + (int64_t)h * S) * 2;
            const float* acc = p.part_acc + (hb + (int64_t)h * S) * D + col;
            float M = NEG_BIG;
            for (int s = sub; s < S; s += L) M = fmaxf(M, ml[2 * s]);
#pragma unroll
            for (int m = 1; m < L; m <<= 1) M = fmaxf(M, __shfl_xor(M, m, 64));
            float num = 0.f, den = 0.f;
            for (int s = sub; s < S; s += L) {
                const float w = fast_exp2(ml[2 * s] - M);
                den = fmaf(w, ml[2 * s + 1], den);
                num = fmaf(w, acc[(int64_t)s * D], num);
            }
#pragma unroll
            for (int m = 1; m < L; m <<= 1) {
                num += __shfl_xor(num, m, 64);
                den += __shfl_xor(den, m, 64);
            }
            if (sub == 0) p.out[(head0 + h) * D + col] = den > 0.f ? num / den : 0.f;
        }
    }
    if (!p.idx) return;         // merge only: nobody will read this layer's index set

    // f(position, key) for every row of the pair: from registers, or re-read from memory
    // (eight independent loads per trip)
    auto for_all_rows = [&](auto&& f) {
        if (ALLREG) {
#pragma unroll
            for (int j = 0; j < NREG; ++j) {
                const int i = grp(j);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (4 * i + e < N) f(4 * i + e, ordered_key(f4_at(v[j], e)));
            }
        } else {
            constexpr int U = 8;
            for (int i0 = tid; i0 < n4; i0 += U * SEL_THREADS) {
                float4 q[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int i = i0 + u * SEL_THREADS;
                    q[u] = i < n4 ? sc4[i] : make_float4(0.f, 0.f, 0.f, 0.f);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int i = i0 + u * SEL_THREADS;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (4 * i + e < N) f(4 * i + e, ordered_key(f4_at(q[u], e)));
                }
            }
        }
    };

    // ---- level 1: threshold bin of the complete histogram ----
    int T1, above1;
    threshold_pick(h4, k, s_wave, s_pick, T1, above1);
    // every thread has consumed its part of the histogram: sign in as one of its C readers
    // (the answer is looked at when the kernel is about to end)
    int arrived = 0;
    if (tid == 0) {
        arrived = __hip_atomic_fetch_add(p.arrive + pair, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_pick[0] = SEL_BINS, s_pick[1] = 0;
    }
    const int kr1 = k - above1;                  // rows of bin T1 that are selected

    // ---- level 2: the rows of bin T1 by their next 12 bits ----
    for_all_rows([&](int, uint32_t key) {
        if ((int)(key >> 20) == T1) atomicAdd(&s_hist[(key >> 8) & (kTopkFineBins - 1)], 1);
    });
    __syncthreads();
    {
#pragma unroll
        for (int e = 0; e < 4; ++e) h4[e] = s_hist[kTopkFineBins - 1 - (4 * tid + e)];
    }
    int T2, above2;
    threshold_pick(h4, kr1, s_wave, s_pick, T2, above2);
    const int kr2 = kr1 - above2;                // rows with the top 24 bits (T1, T2) that are selected
    // (T1 = SEL_BINS when nothing is selected: thr24 is then above every 24-bit value)
    const uint32_t thr24 = ((uint32_t)T1 << 12) | (uint32_t)(T2 & (kTopkFineBins - 1));

    // ---- level 3: rows above the 24-bit threshold are selected; rows equal to it are candidates ----
    int before = 0;                              // selected rows of the chunks before this one
    for_all_rows([&](int pos, uint32_t key) {
        const uint32_t k24 = key >> 8;
        if (k24 > thr24) {
            before += pos < chunk_pos0;
        } else if (k24 == thr24) {
            const int slot = atomicAdd(&s_cand, 1);
            if (slot < SEL_CAP) {
                s_ckey[slot] = key;
                s_cpos[slot] = pos;
            }
        }
    });
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) before += __shfl_xor(before, m, 64);
    if (lane == 0 && before) atomicAdd(&s_before, before);
    __syncthreads();
    const int n_cand = s_cand;

    unsigned long long sel = 0;                  // bit 4 j + e: element e of own register j is selected
    if (n_cand <= SEL_CAP) {
        // exact rank of every candidate under (key descending, position ascending)
        for (int i = tid; i < n_cand; i += SEL_THREADS) {
            const uint32_t key = s_ckey[i];
            const int pos = s_cpos[i];
            int rank = 0;
            for (int j = 0; j < n_cand; ++j) {
                const uint32_t kj = s_ckey[j];
                rank += (kj > key) || (kj == key && s_cpos[j] < pos);
            }
            if (rank < kr2) {
                if (pos < chunk_pos0) atomicAdd(&s_before, 1);
                else if (pos < chunk_pos1) {
                    const int gl = (pos >> 2) - first4;          // owner thread gl % 1024, register gl / 1024
                    atomicOr(&s_sel[gl & (SEL_THREADS - 1)], 1ull << (4 * (gl >> 10) + (pos & 3)));
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < E_OWN; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (4 * grp(j) + e < N && (ordered_key(f4_at(v[j], e)) >> 8) > thr24) sel |= 1ull << (4 * j + e);
        sel |= s_sel[tid];
    } else {
        // rare: more rows share the top 24 key bits than the candidate list holds (massive
        // ties).  Their last 8 bits decide: histogram, threshold key tau, and of the rows
        // equal to tau the first r in position order.
        __syncthreads();
        for (int i = tid; i < 256; i += SEL_THREADS) s_hist[i] = 0;
        __syncthreads();
        for_all_rows([&](int, uint32_t key) {
            if ((key >> 8) == thr24) atomicAdd(&s_hist[key & 255], 1);
        });
        __syncthreads();
        if (tid == 0) {
            int cnt = 0, dg = 255;
            for (; dg > 0; --dg) {
                if (cnt + s_hist[dg] >= kr2) break;
                cnt += s_hist[dg];
            }
            s_kr = kr2 - cnt;
            s_tau = (thr24 << 8) | (uint32_t)dg;
        }
        __syncthreads();
        const uint32_t tau = s_tau;
        const int r = s_kr;
        // rows before this chunk: above tau inside the 24-bit class, and equal to tau
        int gt_b = 0, eq_b = 0;
        for_all_rows([&](int pos, uint32_t key) {
            if (pos < chunk_pos0 && (key >> 8) == thr24) {
                gt_b += key > tau;
                eq_b += key == tau;
            }
        });
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) {
            gt_b += __shfl_xor(gt_b, m, 64);
            eq_b += __shfl_xor(eq_b, m, 64);
        }
        if (lane == 0) {
            if (gt_b) atomicAdd(&s_before, gt_b);
            if (eq_b) atomicAdd(&s_before_eq, eq_b);
        }
        __syncthreads();
        const int eq_before_chunk = s_before_eq;
        unsigned long long eq_mask = 0;
        int eq_cnt[E_OWN], eq_base[E_OWN];
#pragma unroll
        for (int j = 0; j < E_OWN; ++j) {
            eq_cnt[j] = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (4 * grp(j) + e >= N) continue;
                const uint32_t key = ordered_key(f4_at(v[j], e));
                if (key > tau) sel |= 1ull << (4 * j + e);
                else if (key == tau) eq_mask |= 1ull << (4 * j + e), ++eq_cnt[j];
            }
        }
        multi_scan<E_OWN>(eq_cnt, eq_base, s_tot);
#pragma unroll
        for (int j = 0; j < E_OWN; ++j) {
            int seen = eq_before_chunk + eq_base[j];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if ((eq_mask >> (4 * j + e)) & 1) {
                    if (seen < r) sel |= 1ull << (4 * j + e);
                    ++seen;
                }
        }
        if (tid == 0) s_before += min(eq_before_chunk, r);
        __syncthreads();
    }
    const int base0 = s_before;

    // ---- ordered emission of the chunk's selected rows ----
    int cnt[E_OWN], base[E_OWN];
#pragma unroll
    for (int j = 0; j < E_OWN; ++j) cnt[j] = __popc((unsigned)(sel >> (4 * j)) & 0xFu);
    multi_scan<E_OWN>(cnt, base, s_tot);
#pragma unroll
    for (int j = 0; j < E_OWN; ++j) {
        unsigned nib = (unsigned)(sel >> (4 * j)) & 0xFu;
        int o = base0 + base[j];
        const int pos0 = 4 * grp(j);
        while (nib) {
            const int e = __ffs(nib) - 1;
            nib &= nib - 1;
            if (o < k) dst[o] = pos0 + e;
            ++o;
        }
    }

    // ---- the last reader of the pair's histogram leaves it empty ----
    if (tid == 0 && arrived == C - 1) s_last = 1;
    __syncthreads();
    if (s_last) {
        *reinterpret_cast<int4*>(gh + 4 * tid) = make_int4(0, 0, 0, 0);
        if (tid == 0) __hip_atomic_store(p.arrive + pair, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ---- level-1 histogram in a launch of its own, for the streaming kernels that do not bin ----
// grid (chunks of 8192 rows, Hkv, B); the non-empty bins of a chunk are added to the pair's
// histogram with device-scope atomics.
__global__ __launch_bounds__(SEL_THREADS) void score_hist_kernel(TopkParams p) {
    __shared__ int s_hist[SEL_BINS];
    const int c = blockIdx.x, g = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const int64_t pair = (int64_t)b * p.Hkv + g;
    const int N = seq_units(p.seq_lens, b, p.N, p.sel_block);
    const int n4 = (N + 3) >> 2;
    const float4* __restrict__ sc4 = reinterpret_cast<const float4*>(p.scores + pair * p.score_stride);
    float4 v[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int i = (2 * c + j) * SEL_THREADS + tid;
        v[j] = i < n4 ? sc4[i] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    for (int i = tid; i < SEL_BINS; i += SEL_THREADS) s_hist[i] = 0;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (4 * ((2 * c + j) * SEL_THREADS + tid) + e < N) atomicAdd(&s_hist[ordered_key(f4_at(v[j], e)) >> 20], 1);
    __syncthreads();
    int* gh = p.ghist + pair * SEL_BINS;
    for (int i = tid; i < SEL_BINS; i += SEL_THREADS) {
        const int n = s_hist[i];
        if (n) atomicAdd(gh + i, n);
    }
}

hipError_t launch_score_hist(const TopkParams& p, int B, hipStream_t st) {
    const dim3 grid((p.N + 8 * SEL_THREADS - 1) / (8 * SEL_THREADS), p.Hkv, B);
    hipLaunchKernelGGL(score_hist_kernel, grid, dim3(SEL_THREADS), 0, st, p);
    return hipGetLastError();
}

// Rows per chunk are 4096 * e_own; e_all = 0 or the power of two >= ceil(N / 4096) (at most 16)
bool topk_plan(int N, int64_t pairs, int n_cus, int groups, int& e_own, int& e_all) {
    const int64_t n4k = ((int64_t)N + 4095) / 4096;        // float4 groups per thread if one workgroup held all rows
    e_all = 0;
    for (int e = 2; e <= 16; e *= 2)
        if (n4k <= e) {
            e_all = e;
            break;
        }
    if (e_all) {
        // chunks of 8192 rows while that does not launch more than two workgroups per compute
        // unit; else one workgroup per pair
        e_own = (groups == 1 || (groups == 0 && pairs * (e_all / 2) > 2 * (int64_t)n_cus)) ? e_all : 2;
    } else {
        e_own = (groups == 8 || (groups == 0 && pairs * ((n4k + 1) / 2) > 4 * (int64_t)n_cus)) ? 8 : 2;
    }
    return true;
}

hipError_t launch_topk(const TopkParams& p, int B, int e_own, int e_all, hipStream_t st) {
    const int C = (p.N + 4096 * e_own - 1) / (4096 * e_own);
    const dim3 grid(C, p.Hkv, B), block(SEL_THREADS);
#define HYLRA_TOPK(EO, EA)                                                        \
    if (e_own == EO && e_all == EA) {                                             \
        hipLaunchKernelGGL((topk_kernel<EO, EA>), grid, block, 0, st, p);         \
        return hipGetLastError();                                                 \
    }
    HYLRA_TOPK(2, 2) HYLRA_TOPK(2, 4) HYLRA_TOPK(4, 4) HYLRA_TOPK(2, 8) HYLRA_TOPK(8, 8)
    HYLRA_TOPK(2, 16) HYLRA_TOPK(16, 16) HYLRA_TOPK(2, 0) HYLRA_TOPK(8, 0)
#undef HYLRA_TOPK
    return hipErrorInvalidValue;
}

}  // namespace hylra
