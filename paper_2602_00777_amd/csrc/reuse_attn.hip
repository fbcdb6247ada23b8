// Reuse layer (Algorithm 2, Reuse branch): attention over only the KV rows named by the
// inherited index set.  K^sparse / V^sparse are never materialised: each 16-lane or 8-lane
// group of a wave fetches one selected row straight from the cache, and the row serves all
// G query heads of its KV head.  One workgroup handles one slice of the k indices of one
// (batch, KV head) and leaves an online-softmax partial per head for the merge kernel.
#include "attend.h"
#include "launch.h"

namespace hylra {

template <int D, int G, int CH, int R>
__global__ __launch_bounds__(256) void reuse_attn_split_kernel(ReuseParams p) {
    using GEO = Geo<D, G, CH>;
    constexpr int NW = 4;
    constexpr int TILE = R * GEO::RPG;
    __shared__ float smem[merge_smem_floats<GEO, NW>()];

    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunk = lane % GEO::LPR, slot = lane / GEO::LPR;

    const int i0 = split * p.rows_per_split;
    const int i1 = min(p.k, i0 + p.rows_per_split);
    const int32_t* __restrict__ ib = p.idx + ((int64_t)b * p.Hkv + g) * p.k;
    const uint16_t* __restrict__ Kb = p.K + (int64_t)b * p.sb + (int64_t)g * p.sh;
    const uint16_t* __restrict__ Vb = p.V + (int64_t)b * p.sb + (int64_t)g * p.sh;

    uint4 qv[G][CH];
    load_q<GEO>(qv, p.q + ((int64_t)b * p.Hq + (int64_t)g * G) * D, chunk);
    LaneState<GEO> st;
    st.init();

    for (int t0 = i0 + wave * TILE; t0 < i1; t0 += NW * TILE) {
        int64_t off[R];
        bool valid[R];
        float ms[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int pos = t0 + r * GEO::RPG + slot;
            const int row = pos < i1 ? ib[pos] : -1;
            valid[r] = (unsigned)row < (unsigned)p.N;      // negative or >= N: padding, skipped
            off[r] = (int64_t)(valid[r] ? row : 0) * p.sn + chunk * 8;
        }
        attend_tile<GEO, R, true>(st, qv, Kb, Vb, off, valid, p.scale_log2, 0.f, ms);
    }

    const int64_t head0 = (int64_t)b * p.Hq + (int64_t)g * G;
    block_merge_store<GEO, NW>(st, smem, p.part_ml + (head0 * p.n_splits + split) * 2,
                               (int64_t)p.n_splits * 2,
                               p.part_acc + (head0 * p.n_splits + split) * D,
                               (int64_t)p.n_splits * D);
}

template <int D, int G>
struct ReuseCfg {
    static constexpr int CH = (D == 128 && G <= 4) ? 2 : 1;
};

template <int D, int G, int R>
static hipError_t launch_one(const ReuseParams& p, int B, hipStream_t st) {
    dim3 grid(p.n_splits, p.Hkv, B);
    hipLaunchKernelGGL((reuse_attn_split_kernel<D, G, ReuseCfg<D, G>::CH, R>), grid, dim3(256), 0,
                       st, p);
    return hipGetLastError();
}

#define HYLRA_FOR_EACH_G(X, D) X(D, 1) X(D, 2) X(D, 3) X(D, 4) X(D, 5) X(D, 6) X(D, 7) X(D, 8)

int reuse_block_quantum(int D, int G, int variant, int R) {
    if (variant != 0 || (R != 1 && R != 2 && R != 4)) return 0;
#define Q(DD, GG) if (D == DD && G == GG) return 4 * R * Geo<DD, GG, ReuseCfg<DD, GG>::CH>::RPG;
    HYLRA_FOR_EACH_G(Q, 64)
    HYLRA_FOR_EACH_G(Q, 128)
#undef Q
    return 0;
}

hipError_t launch_reuse_split(const ReuseParams& p, int B, int D, int G, int variant, int R,
                              hipStream_t st) {
    if (variant != 0) return hipErrorInvalidValue;
#define L(DD, GG)                                              \
    if (D == DD && G == GG) {                                  \
        if (R == 4) return launch_one<DD, GG, 4>(p, B, st);    \
        if (R == 2) return launch_one<DD, GG, 2>(p, B, st);    \
        if (R == 1) return launch_one<DD, GG, 1>(p, B, st);    \
    }
    HYLRA_FOR_EACH_G(L, 64)
    HYLRA_FOR_EACH_G(L, 128)
#undef L
    return hipErrorInvalidValue;
}

}  // namespace hylra
