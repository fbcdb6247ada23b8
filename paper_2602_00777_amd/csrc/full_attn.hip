// Full layer, streaming pass (Algorithm 2, Full branch): one split of the KV rows of one
// (batch, KV head) per workgroup.  Reads every K and V row of the split exactly once,
// produces per-head online-softmax partials, and the group-mean scaled score of every row
// (the quantity TopK ranks) for the finalise kernel.
#include "attend.h"
#include "launch.h"

namespace hylra {

template <int D, int G, int CH, int R>
__global__ __launch_bounds__(256) void full_attn_split_kernel(FullParams p) {
    using GEO = Geo<D, G, CH>;
    constexpr int NW = 4;
    constexpr int TILE = R * GEO::RPG;
    __shared__ float smem[merge_smem_floats<GEO, NW>()];
    __shared__ float s_mm[2 * NW];

    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunk = lane % GEO::LPR, slot = lane / GEO::LPR;

    const uint16_t* __restrict__ Kb = p.K + (int64_t)b * p.sb + (int64_t)g * p.sh;
    const uint16_t* __restrict__ Vb = p.V + (int64_t)b * p.sb + (int64_t)g * p.sh;
    uint4 qv[G][CH];
    load_q<GEO>(qv, p.q + ((int64_t)b * p.Hq + (int64_t)g * G) * D, chunk);

    LaneState<GEO> st;
    st.init();
    const int row0 = split * p.rows_per_split;
    const int row1 = min(p.N, row0 + p.rows_per_split);
    float* __restrict__ srow = p.scores + ((int64_t)b * p.Hkv + g) * p.score_stride;
    float smin = 3.0e38f, smax = -3.0e38f;

    for (int t0 = row0 + wave * TILE; t0 < row1; t0 += NW * TILE) {
        int64_t off[R];
        bool valid[R];
        float ms[R];
        if (t0 + TILE <= row1) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                off[r] = (int64_t)(t0 + r * GEO::RPG + slot) * p.sn + chunk * 8;
                valid[r] = true;
            }
            attend_tile<GEO, R, false>(st, qv, Kb, Vb, off, valid, p.scale_log2, p.scale_mean, ms);
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const float v = fminf(fmaxf(ms[r], -3.0e38f), 3.0e38f);   // also maps NaN to a number
                if (chunk == 0) srow[t0 + r * GEO::RPG + slot] = v;
                smin = fminf(smin, v);
                smax = fmaxf(smax, v);
            }
        } else {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int row = t0 + r * GEO::RPG + slot;
                valid[r] = row < row1;
                off[r] = (int64_t)(valid[r] ? row : row1 - 1) * p.sn + chunk * 8;
            }
            attend_tile<GEO, R, true>(st, qv, Kb, Vb, off, valid, p.scale_log2, p.scale_mean, ms);
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const float v = fminf(fmaxf(ms[r], -3.0e38f), 3.0e38f);
                if (valid[r]) {
                    if (chunk == 0) srow[t0 + r * GEO::RPG + slot] = v;
                    smin = fminf(smin, v);
                    smax = fmaxf(smax, v);
                }
            }
        }
    }

    // range of this split's group-mean scores (the finalise kernel bins on it)
#pragma unroll
    for (int mask = 1; mask < 64; mask <<= 1) {
        smin = fminf(smin, __shfl_xor(smin, mask, 64));
        smax = fmaxf(smax, __shfl_xor(smax, mask, 64));
    }
    if (lane == 0) {
        s_mm[2 * wave] = smin;
        s_mm[2 * wave + 1] = smax;
    }
    __syncthreads();
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

    const int64_t head0 = (int64_t)b * p.Hq + (int64_t)g * G;
    block_merge_store<GEO, NW>(st, smem, p.part_ml + (head0 * p.n_splits + split) * 2,
                               (int64_t)p.n_splits * 2,
                               p.part_acc + (head0 * p.n_splits + split) * D,
                               (int64_t)p.n_splits * D);
}

// Lane layout per (D, G): two 16-byte pieces per lane while the accumulators still fit a
// two-waves-per-SIMD register budget, one piece for the larger groups.
template <int D, int G>
struct FullCfg {
    static constexpr int CH = (D == 128 && G <= 4) ? 2 : 1;
    static constexpr int R = 4;
};

template <int D, int G>
static hipError_t launch_one(const FullParams& p, int B, hipStream_t st) {
    using C = FullCfg<D, G>;
    dim3 grid(p.n_splits, p.Hkv, B);
    hipLaunchKernelGGL((full_attn_split_kernel<D, G, C::CH, C::R>), grid, dim3(256), 0, st, p);
    return hipGetLastError();
}

template <int D, int G>
static constexpr int quantum_one() {
    using C = FullCfg<D, G>;
    return 4 * C::R * Geo<D, G, C::CH>::RPG;
}

#define HYLRA_FOR_EACH_G(X, D) X(D, 1) X(D, 2) X(D, 3) X(D, 4) X(D, 5) X(D, 6) X(D, 7) X(D, 8)

int full_block_quantum(int D, int G, int variant) {
    if (variant != 0) return 0;
#define Q(DD, GG) if (D == DD && G == GG) return quantum_one<DD, GG>();
    HYLRA_FOR_EACH_G(Q, 64)
    HYLRA_FOR_EACH_G(Q, 128)
#undef Q
    return 0;
}

hipError_t launch_full_split(const FullParams& p, int B, int D, int G, int variant, hipStream_t st) {
    if (variant != 0) return hipErrorInvalidValue;
#define L(DD, GG) if (D == DD && G == GG) return launch_one<DD, GG>(p, B, st);
    HYLRA_FOR_EACH_G(L, 64)
    HYLRA_FOR_EACH_G(L, 128)
#undef L
    return hipErrorInvalidValue;
}

}  // namespace hylra
