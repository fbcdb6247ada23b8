// Full layer, after the streaming pass: merge of the split partials into the attention
// output (Algorithm 2, "O <- Softmax(S) V") and the EXACT selection of the k positions with
// the largest group-mean score (Algorithm 2, "I <- TopK(S, B)"; ties to the lower position,
// ascending order), spread over several workgroups per (batch, KV head).
//
// The scores of one (batch, KV head) are cut into chunks of 4096*E rows; workgroup (c, g, b)
// keeps chunk c in registers.  Three launches, each with grid (C, Hkv, B):
//   1. select_hist_kernel     histogram of the chunk over 4096 equal-width bins spanning the
//                             score range, added into the (batch, KV head)'s global histogram;
//                             also the log-sum-exp merge of the attention partials.
//   2. select_classify_kernel every workgroup finds the threshold bin T from the global
//                             histogram (same result everywhere), counts its rows above T
//                             and appends its rows inside T to a global candidate list.
//   3. select_emit_kernel     every workgroup ranks the candidates (key descending, position
//                             ascending), so it knows which of them are selected, where its
//                             chunk starts in the output, and writes its part of idx.
// If more rows share the threshold bin than the candidate list holds (massive ties), launch 3
// falls back to a radix select over all keys, done redundantly by every workgroup.
// Between launches of a Full layer the global histogram and the candidate count are zero:
// launch 3 clears the histogram, launch 1 the count.
#include "launch.h"
#include "select_util.h"

namespace hylra {

template <int E>
struct Chunk {
    float4 v[E];
    int first4;     // index of the chunk's first float4 group
    int N;
    DEVI void load(const float* sc, int n, int c) {
        N = n;
        first4 = c * E * SEL_THREADS;
        const int n4 = (n + 3) >> 2;
#pragma unroll
        for (int j = 0; j < E; ++j) {
            const int i = first4 + j * SEL_THREADS + (int)threadIdx.x;
            v[j] = i < n4 ? reinterpret_cast<const float4*>(sc)[i] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    // position of element e of this thread's j-th group
    DEVI int pos(int j, int e) const { return 4 * (first4 + j * SEL_THREADS + (int)threadIdx.x) + e; }
    DEVI float at(int j, int e) const {
        return e == 0 ? v[j].x : e == 1 ? v[j].y : e == 2 ? v[j].z : v[j].w;
    }
};

// Range of the group-mean scores of one (batch, KV head) from the per-split ranges, and the
// bin width.  Every workgroup and every launch computes it the same way from the same data.
DEVI void score_range(const SelectParams& p, int64_t pair, float* s_red, float& lo, float& inv_w) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float a = 3.0e38f, b = -3.0e38f;
    const PartView pv = part_view(p.pair_map, pair, p.n_splits);
    for (int s = tid; s < pv.S; s += SEL_THREADS) {
        a = fminf(a, p.part_mm[(pv.first + s) * 2]);
        b = fmaxf(b, p.part_mm[(pv.first + s) * 2 + 1]);
    }
#pragma unroll
    for (int mask = 1; mask < 64; mask <<= 1) {
        a = fminf(a, __shfl_xor(a, mask, 64));
        b = fmaxf(b, __shfl_xor(b, mask, 64));
    }
    if (lane == 0) {
        s_red[2 * wave] = a;
        s_red[2 * wave + 1] = b;
    }
    __syncthreads();
    a = s_red[0];
    b = s_red[1];
#pragma unroll
    for (int w = 1; w < SEL_WAVES; ++w) {
        a = fminf(a, s_red[2 * w]);
        b = fmaxf(b, s_red[2 * w + 1]);
    }
    __syncthreads();
    lo = a;
    const float span = b - a;
    inv_w = (span > 0.f && span < 3.0e38f) ? (float)SEL_BINS / span : 0.f;
}

template <int E>
__global__ __launch_bounds__(SEL_THREADS) void select_hist_kernel(SelectParams p) {
    __shared__ int s_hist[SEL_BINS];
    __shared__ float s_red[2 * SEL_WAVES];
    const int c = blockIdx.x, g = blockIdx.y, b = blockIdx.z, C = gridDim.x;
    const int tid = threadIdx.x;
    const int64_t pair = (int64_t)b * p.Hkv + g;
    const PartView pv = part_view(p.pair_map, pair, p.n_splits);
    const int S = pv.S, D = p.D, G = p.G;
    const int64_t hb = pv.first * G;              // first partial of the pair's first head

    const int N = p.idx ? seq_units(p.seq_lens, b, p.N, p.sel_block) : 0; // rows this sequence ranks (none: merge only)
    Chunk<E> ch;
    ch.load(p.scores + pair * p.score_stride, N, c);        // in flight during the merge below
    for (int i = tid; i < SEL_BINS; i += SEL_THREADS) s_hist[i] = 0;
    if (c == 0 && tid == 0) {
        p.cand_n[pair] = 0;
    }

    // attention output: this workgroup's share of the G*D outputs of the KV head.  16 lanes per
    // output element, each merging every 16th partial (with many partials per head, one thread
    // per element would walk them one after the other while most of the workgroup idles).
    const int share = (G * D + C - 1) / C;
    const int64_t head0 = (int64_t)b * p.Hq + (int64_t)g * G;
    {
        constexpr int L = 16;
        const int sub = tid & (L - 1), grp = tid / L;
        const int end = min(G * D, (c + 1) * share);
        for (int i = c * share + grp; i < end; i += SEL_THREADS / L) {
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
    float lo, inv_w;
    score_range(p, pair, s_red, lo, inv_w);     // its barriers also cover the zeroing above
#pragma unroll
    for (int j = 0; j < E; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (ch.pos(j, e) < N) atomicAdd(&s_hist[score_bin(ch.at(j, e), lo, inv_w)], 1);
    __syncthreads();
    int* gh = p.ghist + pair * SEL_BINS;
    for (int i = tid; i < SEL_BINS; i += SEL_THREADS) {
        const int n = s_hist[i];
        if (n) atomicAdd(gh + i, n);
    }
}

// Threshold bin from the complete histogram: the bin T holding the k-th largest score and
// the number of rows in the bins above it.  Thread t owns bins NB-1-4t ... NB-4-4t.
DEVI void threshold_bin(const int* gh, int k, int* s_wave, int* s_pick, int& T, int& above) {
    const int tid = threadIdx.x;
    int h4[4], local = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        h4[e] = gh[SEL_BINS - 1 - (4 * tid + e)];
        local += h4[e];
    }
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
}

template <int E>
__global__ __launch_bounds__(SEL_THREADS) void select_classify_kernel(SelectParams p) {
    __shared__ float s_red[2 * SEL_WAVES];
    __shared__ int s_wave[SEL_WAVES + 1];
    __shared__ int s_pick[2];
    __shared__ int s_gt;
    const int c = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x;
    const int64_t pair = (int64_t)b * p.Hkv + g;

    const int N = seq_units(p.seq_lens, b, p.N, p.sel_block), k = min(p.k, N);
    Chunk<E> ch;
    ch.load(p.scores + pair * p.score_stride, N, c);
    if (tid == 0) s_gt = 0, s_pick[0] = SEL_BINS, s_pick[1] = 0;      // (k = 0: nothing is selected)
    float lo, inv_w;
    score_range(p, pair, s_red, lo, inv_w);
    int T, above;
    threshold_bin(p.ghist + pair * SEL_BINS, k, s_wave, s_pick, T, above);

    int gt = 0;
#pragma unroll
    for (int j = 0; j < E; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (ch.pos(j, e) >= N) continue;
            const float x = ch.at(j, e);
            const int bn = score_bin(x, lo, inv_w);
            if (bn > T) ++gt;
            else if (bn == T) {
                const int slot = atomicAdd(p.cand_n + pair, 1);
                if (slot < SEL_CAP) {
                    p.cand_key[pair * SEL_CAP + slot] = ordered_key(x);
                    p.cand_pos[pair * SEL_CAP + slot] = ch.pos(j, e);
                }
            }
        }
#pragma unroll
    for (int mask = 1; mask < 64; mask <<= 1) gt += __shfl_xor(gt, mask, 64);
    if ((tid & 63) == 0 && gt) atomicAdd(&s_gt, gt);
    __syncthreads();
    if (tid == 0) {
        p.chunk_gt[pair * p.max_chunks + c] = s_gt;
        if (c == 0) {
            p.sel_info[pair * 2] = T;
            p.sel_info[pair * 2 + 1] = above;
        }
    }
}

template <int E>
__global__ __launch_bounds__(SEL_THREADS) void select_emit_kernel(SelectParams p) {
    __shared__ int s_hist[256];
    __shared__ uint32_t s_ckey[SEL_CAP];
    __shared__ int s_cpos[SEL_CAP];
    __shared__ unsigned long long s_sel[SEL_THREADS];   // candidates of this chunk that made the cut
    __shared__ float s_red[2 * SEL_WAVES];
    __shared__ int s_tot[E * SEL_WAVES + 1];
    __shared__ int s_before, s_before_eq, s_kr;
    __shared__ uint32_t s_tau;
    const int c = blockIdx.x, g = blockIdx.y, b = blockIdx.z, C = gridDim.x;
    const int tid = threadIdx.x;
    const int64_t pair = (int64_t)b * p.Hkv + g;
    const int N = seq_units(p.seq_lens, b, p.N, p.sel_block), k = min(p.k, N);
    const float* __restrict__ sc = p.scores + pair * p.score_stride;
    int32_t* __restrict__ dst = p.idx + pair * (int64_t)p.k;
    if (c == 0)
        for (int i = k + tid; i < p.k; i += SEL_THREADS) dst[i] = -1;  // entries beyond a short sequence

    Chunk<E> ch;
    ch.load(sc, N, c);
    s_sel[tid] = 0;
    if (tid == 0) s_before = 0, s_before_eq = 0;
    float lo, inv_w;
    score_range(p, pair, s_red, lo, inv_w);
    const int T = p.sel_info[pair * 2], above = p.sel_info[pair * 2 + 1];
    const int kr = k - above;                   // rows of bin T that are selected
    const int n_cand = p.cand_n[pair];
    const int chunk_pos0 = 4 * ch.first4, chunk_pos1 = chunk_pos0 + 4 * E * SEL_THREADS;

    // the histogram is complete and no longer read: clear this workgroup's share of it
    {
        int* gh = p.ghist + pair * SEL_BINS;
        const int per = (SEL_BINS + C - 1) / C;
        for (int i = c * per + tid; i < min(SEL_BINS, (c + 1) * per); i += SEL_THREADS) gh[i] = 0;
    }

    // rows of this chunk above the threshold bin; start of the chunk in the output
    int base0 = 0;
    for (int cc = 0; cc < c; ++cc) base0 += p.chunk_gt[pair * p.max_chunks + cc];

    unsigned long long sel = 0;
    if (n_cand <= SEL_CAP) {
        for (int i = tid; i < n_cand; i += SEL_THREADS) {
            s_ckey[i] = p.cand_key[pair * SEL_CAP + i];
            s_cpos[i] = p.cand_pos[pair * SEL_CAP + i];
        }
        __syncthreads();
        for (int i = tid; i < n_cand; i += SEL_THREADS) {
            const uint32_t key = s_ckey[i];
            const int pos = s_cpos[i];
            int rank = 0;
            for (int j = 0; j < n_cand; ++j) {
                const uint32_t kj = s_ckey[j];
                rank += (kj > key) || (kj == key && s_cpos[j] < pos);
            }
            if (rank < kr) {
                if (pos < chunk_pos0) atomicAdd(&s_before, 1);
                else if (pos < chunk_pos1) {
                    const int grp = (pos >> 2) - ch.first4;      // owner thread grp % 1024, slot grp / 1024
                    atomicOr(&s_sel[grp & (SEL_THREADS - 1)], 1ull << (4 * (grp >> 10) + (pos & 3)));
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < E; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (ch.pos(j, e) < N && score_bin(ch.at(j, e), lo, inv_w) > T) sel |= 1ull << (4 * j + e);
        sel |= s_sel[tid];
        base0 += s_before;
    } else {
        // rare: more rows share the threshold bin than the candidate list holds.  Radix select
        // over all keys of the (batch, KV head), 8 bits per pass, done by every workgroup.
        const int n4 = (N + 3) >> 2;
        uint32_t prefix = 0, mask = 0;
        int want = k;
        for (int shift = 24; shift >= 0; shift -= 8) {
            __syncthreads();
            for (int i = tid; i < 256; i += SEL_THREADS) s_hist[i] = 0;
            __syncthreads();
            for (int i = tid; i < n4; i += SEL_THREADS) {
                const float4 q = reinterpret_cast<const float4*>(sc)[i];
                const float x[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t key = ordered_key(x[e]);
                    if (4 * i + e < N && (key & mask) == prefix) atomicAdd(&s_hist[(key >> shift) & 255], 1);
                }
            }
            __syncthreads();
            if (tid == 0) {
                int cnt = 0, dg = 255;
                for (; dg > 0; --dg) {
                    if (cnt + s_hist[dg] >= want) break;
                    cnt += s_hist[dg];
                }
                s_kr = want - cnt;
                s_tau = prefix | ((uint32_t)dg << shift);
            }
            __syncthreads();
            want = s_kr;
            prefix = s_tau;
            mask |= 0xffu << shift;
        }
        const uint32_t tau = prefix;
        const int r = want;          // rows equal to tau that are selected, lowest positions first
        // rows before this chunk: above tau / equal to tau
        int gt_b = 0, eq_b = 0;
        for (int i = tid; i < ch.first4; i += SEL_THREADS) {
            const float4 q = reinterpret_cast<const float4*>(sc)[i];
            const float x[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t key = ordered_key(x[e]);
                gt_b += key > tau;
                eq_b += key == tau;
            }
        }
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) {
            gt_b += __shfl_xor(gt_b, m, 64);
            eq_b += __shfl_xor(eq_b, m, 64);
        }
        if ((tid & 63) == 0) {
            if (gt_b) atomicAdd(&s_before, gt_b);
            if (eq_b) atomicAdd(&s_before_eq, eq_b);
        }
        __syncthreads();
        const int eq_before_chunk = s_before_eq;
        unsigned long long eq_mask = 0;
        int eq_cnt[E], eq_base[E];
#pragma unroll
        for (int j = 0; j < E; ++j) {
            eq_cnt[j] = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (ch.pos(j, e) >= N) continue;
                const uint32_t key = ordered_key(ch.at(j, e));
                if (key > tau) sel |= 1ull << (4 * j + e);
                else if (key == tau) eq_mask |= 1ull << (4 * j + e), ++eq_cnt[j];
            }
        }
        multi_scan<E>(eq_cnt, eq_base, s_tot);
#pragma unroll
        for (int j = 0; j < E; ++j) {
            int seen = eq_before_chunk + eq_base[j];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if ((eq_mask >> (4 * j + e)) & 1) {
                    if (seen < r) sel |= 1ull << (4 * j + e);
                    ++seen;
                }
        }
        base0 = s_before + min(eq_before_chunk, r);
    }

    // ordered emission of the chunk's selected rows
    int cnt[E], base[E];
#pragma unroll
    for (int j = 0; j < E; ++j) cnt[j] = __popc((unsigned)(sel >> (4 * j)) & 0xFu);
    multi_scan<E>(cnt, base, s_tot);
#pragma unroll
    for (int j = 0; j < E; ++j) {
        unsigned nib = (unsigned)(sel >> (4 * j)) & 0xFu;
        int o = base0 + base[j];
        const int pos0 = ch.pos(j, 0);
        while (nib) {
            const int e = __ffs(nib) - 1;
            nib &= nib - 1;
            if (o < k) dst[o] = pos0 + e;
            ++o;
        }
    }
}

int select_chunk_rows(int E) { return 4 * E * SEL_THREADS; }

template <int E>
static hipError_t launch_select_e(const SelectParams& p, int B, int step, hipStream_t st) {
    const int C = (p.N + 4 * E * SEL_THREADS - 1) / (4 * E * SEL_THREADS);
    const dim3 grid(C, p.Hkv, B), block(SEL_THREADS);
    if (step == 0) hipLaunchKernelGGL(select_hist_kernel<E>, grid, block, 0, st, p);
    else if (step == 1) hipLaunchKernelGGL(select_classify_kernel<E>, grid, block, 0, st, p);
    else hipLaunchKernelGGL(select_emit_kernel<E>, grid, block, 0, st, p);
    return hipGetLastError();
}

hipError_t launch_select(const SelectParams& p, int B, int E, int step, hipStream_t st) {
    if (E == 2) return launch_select_e<2>(p, B, step, st);
    if (E == 8) return launch_select_e<8>(p, B, step, st);
    return hipErrorInvalidValue;
}

}  // namespace hylra
