// Full layer, streaming pass (Algorithm 2, Full branch) with the two contractions of Eq. 1 on
// the matrix cores (see mfma_core.h for how a wave consumes 16 rows).  Same role, same
// outputs and same launch geometry as the vector kernel in full_attn_impl.h: per-head
// online-softmax partials, the group-mean score of every row, and their range per split.
// It exists for the larger groups: from G = 5 the vector kernel is bound by its own
// arithmetic, not by HBM (removing its accumulate step alone makes it 20 % faster at G = 7),
// while the matrix cores take that arithmetic off the vector pipeline.
#include "launch.h"
#include "mfma_core.h"

namespace hylra {

template <int D, int NB>
struct MfmaTile {
    uint4 k[NB][D / 32];
    uint4 v[NB][D / 32];
};

// PIPE: two register tiles, the loads of tile i+1 in flight while tile i is consumed.
template <int D, int G, int NB, bool PIPE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void full_mfma_kernel(FullParams p) {
    constexpr int NW = 4;
    constexpr int KI = D / 32;
    constexpr int TILE = 16 * NB;
    __shared__ float s_m[NW][16];
    __shared__ float s_l[NW][16];
    __shared__ float s_acc[NW * G * D];

    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, gq = lane >> 4;

    const bool paged = p.map.table != nullptr;
    const int64_t base = (paged ? 0 : (int64_t)b * p.sb) + (int64_t)g * p.sh;
    const uint16_t* __restrict__ Kb = p.K + base;
    const uint16_t* __restrict__ Vb = p.V + base;
    const int64_t head0 = (int64_t)b * p.Hq + (int64_t)g * G;
    uint4 qb[KI], sel[2];
    mfma_load_q<D, G>(qb, p.q + head0 * D, n, gq);
    mfma_selectors(sel, n, gq);
    MfmaState<D> st;
    st.init();

    constexpr int STEP = NW * TILE;
    // rows of this sequence; a shorter sequence is cut into the same number of (shorter) splits
    const int n_rows = seq_rows(p.map, b, p.N);
    const int rps = n_rows == p.N ? p.rows_per_split
                                  : (n_rows + p.n_splits * STEP - 1) / (p.n_splits * STEP) * STEP;
    const int row0 = split * rps;
    const int row1 = min(n_rows, row0 + rps);
    float* __restrict__ srow = p.scores + ((int64_t)b * p.Hkv + g) * p.score_stride;

    // paged cache: the split's part of the sequence's page table, staged in LDS
    extern __shared__ int s_tbl[];
    // (read from memory if it does not fit there)
    const int32_t* __restrict__ tbl = p.map.table + (int64_t)b * p.map.table_stride;     // unused unless paged
    int tbl_page0 = -1;                                                     // first staged page; -1: not staged
    if (paged && row0 < row1) {
        const int page0 = row0 >> p.map.page_shift, n_pages = ((row1 - 1) >> p.map.page_shift) - page0 + 1;
        if (n_pages <= p.tbl_cap) {
            for (int i = tid; i < n_pages; i += NW * 64) s_tbl[i] = tbl[page0 + i];
            tbl_page0 = page0;
        }
        __syncthreads();
    }
    auto row_offset = [&](int row) -> int64_t {
        if (!paged) return (int64_t)row * p.sn;
        const int t = row >> p.map.page_shift;
        const int page = tbl_page0 >= 0 ? s_tbl[t - tbl_page0] : tbl[t];
        return (int64_t)page * p.map.stride_page + (int64_t)(row & ((1 << p.map.page_shift) - 1)) * p.sn;
    };

    // rows past the end of the split are clamped to its last row and masked when consumed
    auto issue = [&](MfmaTile<D, NB>& buf, int t0) {
#pragma unroll
        for (int blk = 0; blk < NB; ++blk) {
            const int row = min(t0 + 16 * blk + n, row1 - 1);
            const int64_t off = row_offset(row) + 8 * gq;
#pragma unroll
            for (int i = 0; i < KI; ++i) buf.k[blk][i] = ld16<true>(Kb + off + 32 * i);
#pragma unroll
            for (int i = 0; i < KI; ++i) buf.v[blk][i] = ld16<true>(Vb + off + 32 * i);
        }
    };
    auto consume = [&](const MfmaTile<D, NB>& buf, int t0) {
#pragma unroll
        for (int blk = 0; blk < NB; ++blk) {
            const int r0 = t0 + 16 * blk;
            const int left = row1 - r0;                      // rows of this block inside the split
            const uint32_t vmask = left >= 16 ? 0xffffu : left > 0 ? (1u << left) - 1u : 0u;
            const float4_t S = mfma_block<D, G>(st, buf.k[blk], buf.v[blk], qb, sel, vmask, p.scale_log2, n, gq);
            // group-mean score of rows 4 gq + j: sum over the 16 head lanes (padding heads hold 0)
            float sj[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float v = group_sum<16>(S[j]) * p.scale_mean;
                sj[j] = fminf(fmaxf(v, -3.0e38f), 3.0e38f);  // also maps NaN to a number
            }
            if (left >= 16) {
                if (n == 0) *reinterpret_cast<float4*>(srow + r0 + 4 * gq) = make_float4(sj[0], sj[1], sj[2], sj[3]);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (4 * gq + j < left && n == 0) srow[r0 + 4 * gq + j] = sj[j];
            }
        }
    };

    if (!PIPE) {
        for (int t0 = row0 + wave * TILE; t0 < row1; t0 += STEP) {
            MfmaTile<D, NB> buf;
            issue(buf, t0);
            consume(buf, t0);
        }
    } else {
        MfmaTile<D, NB> bufA, bufB;
        int t0 = row0 + wave * TILE;
        if (t0 < row1) issue(bufA, t0);
        while (t0 < row1) {
            if (t0 + STEP < row1) issue(bufB, t0 + STEP);
            consume(bufA, t0);
            t0 += STEP;
            if (t0 >= row1) break;
            if (t0 + STEP < row1) issue(bufA, t0 + STEP);
            consume(bufB, t0);
            t0 += STEP;
        }
    }

    mfma_block_merge_store<D, G, NW, false>(st, s_m, s_l, s_acc,
                                            p.part_ml + (head0 * p.n_splits + split) * 2,
                                            (int64_t)p.n_splits * 2,
                                            p.part_acc + (head0 * p.n_splits + split) * D,
                                            (int64_t)p.n_splits * D, n, gq);
}

// variant = 10 * mode + NB: mode 5 = one tile at a time, mode 6 = two-deep register pipeline
#define HYLRA_FULL_MFMA_VARIANTS(X) X(5, 2, false)

template <int D, int G>
static hipError_t launch_g(const FullParams& p, int B, int variant, hipStream_t st) {
    dim3 grid(p.n_splits, p.Hkv, B);
#define V(MODE, NB, PIPE)                                                                        \
    if (variant == 10 * MODE + NB) {                                                             \
        hipLaunchKernelGGL((full_mfma_kernel<D, G, NB, PIPE>), grid, dim3(256),                  \
                           p.tbl_cap * sizeof(int), st, p);                                      \
        return hipGetLastError();                                                                \
    }
    HYLRA_FULL_MFMA_VARIANTS(V)
#undef V
    return hipErrorInvalidValue;
}

int full_mfma_quantum(int variant) {
#define V(MODE, NB, PIPE) if (variant == 10 * MODE + NB) return 4 * 16 * NB;
    HYLRA_FULL_MFMA_VARIANTS(V)
#undef V
    return 0;
}

hipError_t launch_full_mfma(const FullParams& p, int B, int D, int G, int variant, hipStream_t st) {
#define HYLRA_G(GG)                                                    \
    if (G == GG) {                                                     \
        if (D == 128) return launch_g<128, GG>(p, B, variant, st);     \
        if (D == 64) return launch_g<64, GG>(p, B, variant, st);       \
    }
    HYLRA_G(1) HYLRA_G(2) HYLRA_G(3) HYLRA_G(4) HYLRA_G(5) HYLRA_G(6) HYLRA_G(7) HYLRA_G(8)
#undef HYLRA_G
    return hipErrorInvalidValue;
}

}  // namespace hylra
