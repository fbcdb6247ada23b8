// Full layer, streaming pass (Algorithm 2, Full branch): one split of the KV rows of one
// (batch, KV head) per workgroup.  Reads every K and V row of the split exactly once,
// produces per-head online-softmax partials, and the group-mean scaled score of every row
// (the quantity TopK ranks) for the finalise kernel.
#pragma once
#include "attend.h"
#include "launch.h"

#ifndef HYLRA_BUILD_D
#error "define HYLRA_BUILD_D to 64 or 128"
#endif

namespace hylra {

// MODE 0: plain loads, one tile at a time.  MODE 1: streaming (non-temporal) loads.
// MODE 2: streaming loads and a two-deep register pipeline -- the loads of tile i+1 are
// issued before tile i is consumed, so every wave always has one to two tiles in flight.
//
// The group-mean scores of the split are staged in LDS (rows_per_split floats of dynamic
// shared memory) and written out once, after the loop.  Besides turning them into full
// 16-byte stores this keeps vector stores out of the loop: loads and stores share one
// completion counter on this architecture and do not complete in order with respect to each
// other, so with a store pending every wait for a tile would have to drain the counter to
// zero, i.e. also wait for the tile that was only just requested.  For the same reason the
// pipelined loop issues its look-ahead loads unconditionally (rows past the split are
// clamped to its last row): the number of younger loads at each wait is then a constant.
template <int D, int G, int CH, int R, int MODE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void full_attn_split_kernel(FullParams p) {
    using GEO = Geo<D, G, CH>;
    constexpr int NW = 4;
    constexpr int TILE = R * GEO::RPG;
    constexpr bool NT = MODE >= 1;
    __shared__ float smem[merge_smem_floats<GEO, NW>()];
    __shared__ float s_mm[2 * NW];
    extern __shared__ float s_scores[];          // [rows_per_split]

    const int split = (blockIdx.x + p.split_rot) % p.n_splits, g = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunk = lane % GEO::LPR, slot = lane / GEO::LPR;

    HYLRA_TS(0);
    const uint16_t* __restrict__ Kb = p.K + (int64_t)b * p.sb + (int64_t)g * p.sh;
    const uint16_t* __restrict__ Vb = p.V + (int64_t)b * p.sb + (int64_t)g * p.sh;
    uint4 qv[G][CH];
    load_q<GEO>(qv, p.q + ((int64_t)b * p.Hq + (int64_t)g * G) * D, chunk);

    LaneState<GEO> st;
    st.init();
    const int row0 = split * p.rows_per_split;
    const int row1 = min(p.N, row0 + p.rows_per_split);
    float smin = 3.0e38f, smax = -3.0e38f;

    // element offsets of this lane's rows in the tile starting at row t0 (rows past the end
    // of the split are clamped to its last row; they are masked when consumed)
    auto offsets = [&](int t0, int64_t (&off)[R]) {
#pragma unroll
        for (int r = 0; r < R; ++r)
            off[r] = (int64_t)min(t0 + r * GEO::RPG + slot, row1 - 1) * p.sn + chunk * 8;
    };
    // softmax/accumulate a loaded tile, stage its group-mean scores, track their range
    auto consume = [&](const TileBuf<GEO, R>& buf, int t0) {
        bool valid[R];
        float ms[R];
        if (t0 + TILE <= row1) {
#pragma unroll
            for (int r = 0; r < R; ++r) valid[r] = true;
            compute_tile<GEO, R, false>(st, qv, buf, valid, p.scale_log2, p.scale_mean, ms);
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const float v = fminf(fmaxf(ms[r], -3.0e38f), 3.0e38f);   // also maps NaN to a number
                if (chunk == 0) s_scores[t0 - row0 + r * GEO::RPG + slot] = v;
                smin = fminf(smin, v);
                smax = fmaxf(smax, v);
            }
        } else {
#pragma unroll
            for (int r = 0; r < R; ++r) valid[r] = t0 + r * GEO::RPG + slot < row1;
            compute_tile<GEO, R, true>(st, qv, buf, valid, p.scale_log2, p.scale_mean, ms);
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const float v = fminf(fmaxf(ms[r], -3.0e38f), 3.0e38f);
                if (valid[r]) {
                    if (chunk == 0) s_scores[t0 - row0 + r * GEO::RPG + slot] = v;
                    smin = fminf(smin, v);
                    smax = fmaxf(smax, v);
                }
            }
        }
    };

    constexpr int STEP = NW * TILE;
    if (MODE < 2) {
        for (int t0 = row0 + wave * TILE; t0 < row1; t0 += STEP) {
            int64_t off[R];
            TileBuf<GEO, R> buf;
            offsets(t0, off);
            load_tile<GEO, R, NT>(buf, Kb, Vb, off);
            consume(buf, t0);
        }
    } else {
        TileBuf<GEO, R> bufA, bufB;
        int64_t off[R];
        int t0 = row0 + wave * TILE;
        offsets(t0, off);
        load_tile<GEO, R, NT>(bufA, Kb, Vb, off);
        while (t0 < row1) {
            offsets(t0 + STEP, off);
            load_tile<GEO, R, NT>(bufB, Kb, Vb, off);
            consume(bufA, t0);
            t0 += STEP;
            if (t0 >= row1) break;
            offsets(t0 + STEP, off);
            load_tile<GEO, R, NT>(bufA, Kb, Vb, off);
            consume(bufB, t0);
            t0 += STEP;
        }
    }

    HYLRA_TS(1);
    // range of this split's group-mean scores (the finalise kernel bins on it)
    smin = strided_minmax<1, false>(smin);
    smax = strided_minmax<1, true>(smax);
    if (lane == 0) {
        s_mm[2 * wave] = smin;
        s_mm[2 * wave + 1] = smax;
    }
    __syncthreads();                             // also: every score of the split is in LDS
    if (tid == 0) {
#pragma unroll
        for (int w = 1; w < NW; ++w) {
            smin = fminf(smin, s_mm[2 * w]);
            smax = fmaxf(smax, s_mm[2 * w + 1]);
        }
        float* mm = p.part_mm + (((int64_t)b * p.Hkv + g) * p.n_splits + split) * 2;
        mm[0] = smin;
        mm[1] = smax;
    }
    {
        // row0 and the score stride are multiples of 4 floats: 16-byte stores are aligned
        float* __restrict__ dst = p.scores + ((int64_t)b * p.Hkv + g) * p.score_stride + row0;
        const int n = row1 - row0;
        for (int i = 4 * tid; i < n; i += 4 * NW * 64) {
            if (i + 4 <= n) {
                *reinterpret_cast<float4*>(dst + i) = *reinterpret_cast<const float4*>(s_scores + i);
            } else {
                for (int e = i; e < n; ++e) dst[e] = s_scores[e];
            }
        }
    }

    const int64_t head0 = (int64_t)b * p.Hq + (int64_t)g * G;
    block_merge_store<GEO, NW>(st, smem, p.part_ml + (head0 * p.n_splits + split) * 2,
                               (int64_t)p.n_splits * 2,
                               p.part_acc + (head0 * p.n_splits + split) * D,
                               (int64_t)p.n_splits * D);
    HYLRA_TS(2);
}

// Lane layout per (D, G): two 16-byte pieces per lane while the accumulators still fit a
// two-waves-per-SIMD register budget, one piece for the larger groups.
template <int D, int G>
struct FullCfg {
    static constexpr int CH = (D == 128 && G <= 4) ? 2 : 1;
};

// variant = 10 * MODE + R  (R = row groups per tile)
#define HYLRA_FULL_VARIANTS(X) X(0, 4) X(1, 4) X(2, 3)
constexpr int kDefaultFullVariant = 23;

template <int D, int G>
static hipError_t launch_one(const FullParams& p, int B, int variant, hipStream_t st) {
    constexpr int CH = FullCfg<D, G>::CH;
    dim3 grid(p.n_splits, p.Hkv, B);
#define V(MODE, R)                                                                              \
    if (variant == 10 * MODE + R) {                                                             \
        hipLaunchKernelGGL((full_attn_split_kernel<D, G, CH, R, MODE>), grid, dim3(256),        \
                           p.rows_per_split * sizeof(float), st, p);                            \
        return hipGetLastError();                                                               \
    }
    HYLRA_FULL_VARIANTS(V)
#undef V
    return hipErrorInvalidValue;
}

static bool variant_known(int variant) {
#define V(MODE, R) if (variant == 10 * MODE + R) return true;
    HYLRA_FULL_VARIANTS(V)
#undef V
    return false;
}

#define HYLRA_FOR_EACH_G(X, D) X(D, 1) X(D, 2) X(D, 3) X(D, 4) X(D, 5) X(D, 6) X(D, 7) X(D, 8)

#if HYLRA_BUILD_D == 64
#define HYLRA_SUFFIX(name) name##_d64
#else
#define HYLRA_SUFFIX(name) name##_d128
#endif

int HYLRA_SUFFIX(full_block_quantum)(int G, int variant) {
    if (variant == 0) variant = kDefaultFullVariant;
    if (!variant_known(variant)) return 0;
    const int R = variant % 10;
#define Q(DD, GG) if (G == GG) return 4 * R * Geo<DD, GG, FullCfg<DD, GG>::CH>::RPG;
    HYLRA_FOR_EACH_G(Q, HYLRA_BUILD_D)
#undef Q
    return 0;
}

hipError_t HYLRA_SUFFIX(launch_full_split)(const FullParams& p, int B, int G, int variant, hipStream_t st) {
    if (variant == 0) variant = kDefaultFullVariant;
#define L(DD, GG) if (G == GG) return launch_one<DD, GG>(p, B, variant, st);
    HYLRA_FOR_EACH_G(L, HYLRA_BUILD_D)
#undef L
    return hipErrorInvalidValue;
}

}  // namespace hylra
