// Reuse layer (Algorithm 2, Reuse branch): attention over only the KV rows named by the
// inherited index set.  K^sparse / V^sparse are never materialised: each 8- or 16-lane
// group of a wave fetches one selected row straight from the cache, and the row serves all
// G query heads of its KV head.  One workgroup handles one slice of the k indices of one
// (batch, KV head) and leaves an online-softmax partial per head; the workgroup that
// finishes last for a (batch, KV head) merges the partials into the output (or, in the
// unfused mode, a separate merge kernel does).
#pragma once
#include "attend.h"
#include "launch.h"
#include "reuse_tail.h"

#ifndef HYLRA_BUILD_D
#error "define HYLRA_BUILD_D to 64 or 128"
#endif

namespace hylra {

template <int D, int G, int CH, int R, bool NT>
__global__ __launch_bounds__(256) void reuse_attn_split_kernel(ReuseParams p) {
    using GEO = Geo<D, G, CH>;
    constexpr int NW = 4;
    constexpr int TILE = R * GEO::RPG;
    __shared__ float smem[merge_smem_floats<GEO, NW>()];
    __shared__ int s_last;

    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunk = lane % GEO::LPR, slot = lane / GEO::LPR;

    // rows of this sequence (entries that name a row beyond them are padding); with none,
    // nothing is loaded
    const int n_rows = seq_rows(p.map, b, p.N);
    const int i0 = split * p.rows_per_split;
    const int i1 = n_rows > 0 ? min(p.k, i0 + p.rows_per_split) : i0;
    const int64_t pair = (int64_t)b * p.Hkv + g;
    const int32_t* __restrict__ ib = p.idx + pair * p.idx_stride;
    const int32_t* __restrict__ tbl = p.map.table ? p.map.table + (int64_t)b * p.map.table_stride : nullptr;
    const int64_t base = (tbl ? 0 : (int64_t)b * p.sb) + (int64_t)g * p.sh;
    const uint16_t* __restrict__ Kb = p.K + base;
    const uint16_t* __restrict__ Vb = p.V + base;

    HYLRA_TS(0);
    // the index loads head the longest dependent chain (index -> row -> softmax): issue first
    int t0 = i0 + wave * TILE;
    int row[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int pos = t0 + r * GEO::RPG + slot;
        row[r] = pos < i1 ? reuse_row(p, ib, pos) : -1;
    }
    uint4 qv[G][CH];
    load_q<GEO>(qv, p.q + ((int64_t)b * p.Hq + (int64_t)g * G) * D, chunk);
    LaneState<GEO> st;
    st.init();

    // A tile is issued as SUB sub-tiles of RS row groups (K rows then V rows of each), all
    // loads up front, and consumed sub-tile by sub-tile: the softmax of the first rows runs
    // while the later rows are still in flight.
    constexpr int RS = R < 2 ? R : 2;
    constexpr int SUB = R / RS;
    while (t0 < i1) {
        HYLRA_TS(1);
        TileBuf<GEO, RS> buf[SUB];
        bool valid[SUB][RS];
#pragma unroll
        for (int u = 0; u < SUB; ++u) {
            int64_t off[RS];
#pragma unroll
            for (int r = 0; r < RS; ++r) {
                const int rr = row[u * RS + r];
                valid[u][r] = (unsigned)rr < (unsigned)n_rows;  // negative or past the sequence: padding, skipped
                off[r] = reuse_row_offset(p, tbl, valid[u][r] ? rr : 0) + chunk * 8;
            }
            load_tile<GEO, RS, NT>(buf[u], Kb, Vb, off);
        }
        t0 += NW * TILE;
        if (t0 < i1) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int pos = t0 + r * GEO::RPG + slot;
                row[r] = pos < i1 ? reuse_row(p, ib, pos) : -1;
            }
        }
#pragma unroll
        for (int u = 0; u < SUB; ++u) {
            float ms[RS];
            compute_tile<GEO, RS, true>(st, qv, buf[u], valid[u], p.scale_log2, 0.f, ms);
        }
        HYLRA_TS(2);
    }

    const int64_t head0 = (int64_t)b * p.Hq + (int64_t)g * G;
    float* const my_ml = p.part_ml + (head0 * p.n_splits + split) * 2;
    float* const my_acc = p.part_acc + (head0 * p.n_splits + split) * D;
    if (p.counters == nullptr) {            // unfused: a separate kernel merges the partials
        block_merge_store<GEO, NW, false>(st, smem, my_ml, (int64_t)p.n_splits * 2, my_acc,
                                          (int64_t)p.n_splits * D);
        return;
    }

    // Fused merge: partials go out with device-scope write-through stores; once they are
    // complete the workgroup bumps the arrival counter of its (batch, KV head); whoever
    // arrives last reads all partials back with device-scope loads and writes the output.
    block_merge_store<GEO, NW, true>(st, smem, my_ml, (int64_t)p.n_splits * 2, my_acc,
                                     (int64_t)p.n_splits * D);
    reuse_merge_tail<G, D, NW * 64>(p, pair, head0, &s_last);
}

template <int D, int G>
struct ReuseCfg {
    static constexpr int CH = (D == 128 && G <= 4) ? 2 : 1;
};

template <int D, int G, int R>
static hipError_t launch_r(const ReuseParams& p, int B, int variant, hipStream_t st) {
    constexpr int CH = ReuseCfg<D, G>::CH;
    dim3 grid(p.n_splits, p.Hkv, B);
    if (variant == 1)
        hipLaunchKernelGGL((reuse_attn_split_kernel<D, G, CH, R, false>), grid, dim3(256), 0, st, p);
    else
        hipLaunchKernelGGL((reuse_attn_split_kernel<D, G, CH, R, true>), grid, dim3(256), 0, st, p);
    return hipGetLastError();
}

#define HYLRA_FOR_EACH_G(X, D) X(D, 1) X(D, 2) X(D, 3) X(D, 4) X(D, 5) X(D, 6) X(D, 7) X(D, 8)

#if HYLRA_BUILD_D == 64
#define HYLRA_SUFFIX(name) name##_d64
#else
#define HYLRA_SUFFIX(name) name##_d128
#endif

// variant 0 = streaming (non-temporal) loads, 1 = plain loads
int HYLRA_SUFFIX(reuse_block_quantum)(int G, int variant, int R) {
    if (variant < 0 || variant > 1 || (R != 1 && R != 2 && R != 4 && R != 8)) return 0;
#define Q(DD, GG) if (G == GG) return 4 * R * Geo<DD, GG, ReuseCfg<DD, GG>::CH>::RPG;
    HYLRA_FOR_EACH_G(Q, HYLRA_BUILD_D)
#undef Q
    return 0;
}

hipError_t HYLRA_SUFFIX(launch_reuse_split)(const ReuseParams& p, int B, int G, int variant, int R,
                                            hipStream_t st) {
    if (variant < 0 || variant > 1) return hipErrorInvalidValue;
#define L(DD, GG)                                                   \
    if (G == GG) {                                                  \
        if (R == 8) return launch_r<DD, GG, 8>(p, B, variant, st);  \
        if (R == 4) return launch_r<DD, GG, 4>(p, B, variant, st);  \
        if (R == 2) return launch_r<DD, GG, 2>(p, B, variant, st);  \
        if (R == 1) return launch_r<DD, GG, 1>(p, B, variant, st);  \
    }
    HYLRA_FOR_EACH_G(L, HYLRA_BUILD_D)
#undef L
    return hipErrorInvalidValue;
}

}  // namespace hylra
