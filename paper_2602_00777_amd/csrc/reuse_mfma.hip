// Reuse layer (Algorithm 2, Reuse branch) with the two contractions of Eq. 1 on the matrix
// cores.  Same decomposition and same cross-workgroup merge as the vector kernel
// (reuse_attn_impl.h); what differs is how one wave consumes a block of 16 gathered rows:
//
//   scores   S[r][h] = K[r][:] . q[h][:]            v_mfma_f32_16x16x32_bf16, A = K rows as
//            loaded (lane = row, 8 consecutive columns per register quad), B = q with the G
//            heads padded to 16 columns.  bf16 products are exact, accumulation is fp32.
//            The result sits as lane = head, registers = 4 rows: exactly the A-operand shape
//            the second contraction wants for the weights.
//   V^T      the PV contraction runs over rows, but a gathered V row is column-contiguous.
//            A 16x32 V tile is pushed through one more MFMA against a constant 0/1 selector,
//            which returns it as lane = column, registers = 4 rows (exact, values stay bf16):
//            the B-operand shape of a 16x16x16 MFMA.  No LDS round trip.
//   output   acc[h][c] += P[h][r] V[r][c]            v_mfma_f32_16x16x16_bf16, with the fp32
//            weight split into a high and a low bf16 part (two MFMAs), so the weights carry
//            16 mantissa bits.
//
// Why matrix cores here although the group is only G <= 8 rows of a 16-row tile: with the
// vector kernel the softmax/accumulate arithmetic of a Reuse layer (about 0.27 GFLOP) costs
// about 4 us of a 21 us kernel that moves only 64 MiB, and it is exposed, not hidden (timed
// by removing it); for G > 4 the same arithmetic also limits the streaming Full kernel.
#include "launch.h"
#include "mfma_core.h"
#include "reuse_tail.h"

namespace hylra {

// NB blocks of 16 rows per wave tile, NW waves per workgroup.  With 8 waves one workgroup fills
// a compute unit (two waves per SIMD), so all waves of the unit start together and issue their
// index loads before any row load is queued in the unit's memory pipeline; with 4 waves the
// second workgroup of a unit can find its index loads queued behind the first one's rows.
template <int D, int G, int NB, bool NT, int NW>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2))) void reuse_mfma_kernel(ReuseParams p) {
    constexpr int KI = D / 32;          // 32-column steps of the score contraction
    constexpr int ROWS_W = 16 * NB;
    __shared__ float s_m[NW][16];
    __shared__ float s_l[NW][16];
    __shared__ float s_acc[NW * G * D];
    __shared__ int s_last;

    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, gq = lane >> 4;

    // rows of this sequence (entries that name a row beyond them are padding); with none,
    // nothing is loaded
    int n_rows = seq_rows(p.map, b, p.N);
    const int64_t pair = (int64_t)b * p.Hkv + g;
    const NewRow nr = reuse_new_row<D>(p, b, pair, n_rows);
    const int i0 = split * p.rows_per_split;
    const int i1 = n_rows > 0 ? min(p.k, i0 + p.rows_per_split) : i0;
    const int64_t head0 = (int64_t)b * p.Hq + (int64_t)g * G;
    const int32_t* __restrict__ ib = p.idx + pair * p.idx_stride;
    const int32_t* __restrict__ tbl = p.map.table ? p.map.table + (int64_t)b * p.map.table_stride : nullptr;
    const int64_t base = (tbl ? 0 : (int64_t)b * p.sb) + (int64_t)g * p.sh;
    const uint16_t* __restrict__ Kb = p.K + base;
    const uint16_t* __restrict__ Vb = p.V + base;

    reuse_store_new_row<D>(p, nr, tbl, Kb, Vb, split, tid);

    HYLRA_TS(0);
    // the index loads head the longest dependent chain (index -> row -> softmax): issue first
    int t0 = i0 + wave * ROWS_W;
    int row[NB];
#pragma unroll
    for (int blk = 0; blk < NB; ++blk) {
        const int pos = t0 + 16 * blk + n;
        row[blk] = pos < i1 ? reuse_row(p, ib, pos) : -1;
    }
    uint4 qb[KI], sel[2];
    mfma_load_q<D, G>(qb, p.q + head0 * D, n, gq);
    mfma_selectors(sel, n, gq);
    MfmaState<D> st;
    st.init();

    while (t0 < i1) {
        HYLRA_TS(1);
        uint4 kb[NB][KI], vb[NB][KI];
        bool valid[NB];
#pragma unroll
        for (int blk = 0; blk < NB; ++blk) {
            valid[blk] = (unsigned)row[blk] < (unsigned)n_rows;    // negative or past the sequence: padding
            const int r = valid[blk] ? row[blk] : 0;
            const int64_t off = reuse_row_offset(p, tbl, r);
            // (the token being appended is not in the cache yet)
            const uint16_t* kp = (r == nr.row ? nr.k : Kb + off) + 8 * gq;
            const uint16_t* vp = (r == nr.row ? nr.v : Vb + off) + 8 * gq;
#pragma unroll
            for (int i = 0; i < KI; ++i) kb[blk][i] = ld16<NT>(kp + 32 * i);
#pragma unroll
            for (int i = 0; i < KI; ++i) vb[blk][i] = ld16<NT>(vp + 32 * i);
        }
        t0 += NW * ROWS_W;
        if (t0 < i1) {
#pragma unroll
            for (int blk = 0; blk < NB; ++blk) {
                const int pos = t0 + 16 * blk + n;
                row[blk] = pos < i1 ? reuse_row(p, ib, pos) : -1;
            }
        }
#pragma unroll
        for (int blk = 0; blk < NB; ++blk) {
            // lanes 0..15 carry the 16 rows' validity
            const uint32_t vmask = (uint32_t)__builtin_amdgcn_ballot_w64(valid[blk]) & 0xffffu;
            mfma_block<D, G>(st, kb[blk], vb[blk], qb, sel, vmask, p.scale_log2, n, gq);
        }
        HYLRA_TS(2);
    }

    float* const my_ml = p.part_ml + (head0 * p.n_splits + split) * 2;
    float* const my_acc = p.part_acc + (head0 * p.n_splits + split) * D;
    const int64_t ml_stride = (int64_t)p.n_splits * 2, acc_stride = (int64_t)p.n_splits * D;
    if (p.n_splits == 1 && p.counters) {    // nothing crosses workgroups: no partial, no counter
        mfma_stage_states<D, G, NW>(st, s_m, s_l, s_acc, n, gq);
        staged_to_output<D, G, NW>(s_m, s_l, s_acc, p.out + head0 * D);
        return;
    }
    if (p.counters == nullptr) {            // unfused: a separate kernel merges the partials
        mfma_block_merge_store<D, G, NW, false>(st, s_m, s_l, s_acc, my_ml, ml_stride, my_acc, acc_stride, n, gq);
        return;
    }
    mfma_block_merge_store<D, G, NW, true>(st, s_m, s_l, s_acc, my_ml, ml_stride, my_acc, acc_stride, n, gq);
    reuse_merge_tail<G, D, NW * 64>(p, pair, head0, &s_last);
}

template <int D, int G>
static hipError_t launch_g(const ReuseParams& p, int B, int NB, bool nt, int NW, hipStream_t st) {
    dim3 grid(p.n_splits, p.Hkv, B);
#define HYLRA_MFMA_CASE(NBV, NWV)                                                                              \
    if (NB == NBV && NW == NWV) {                                                                              \
        if (nt) hipLaunchKernelGGL((reuse_mfma_kernel<D, G, NBV, true, NWV>), grid, dim3(NWV * 64), 0, st, p); \
        else hipLaunchKernelGGL((reuse_mfma_kernel<D, G, NBV, false, NWV>), grid, dim3(NWV * 64), 0, st, p);   \
        return hipGetLastError();                                                                              \
    }
    HYLRA_MFMA_CASE(4, 4)
    HYLRA_MFMA_CASE(2, 4)
    HYLRA_MFMA_CASE(1, 4)
    HYLRA_MFMA_CASE(4, 8)
#undef HYLRA_MFMA_CASE
    return hipErrorInvalidValue;
}

// rows per workgroup sweep with NB blocks of 16 rows per wave and NW waves
int reuse_mfma_quantum(int NB, int NW) {
    const bool ok = (NW == 4 && (NB == 1 || NB == 2 || NB == 4)) || (NW == 8 && NB == 4);
    return ok ? NW * 16 * NB : 0;
}

hipError_t launch_reuse_mfma(const ReuseParams& p, int B, int D, int G, int NB, bool nt, int NW, hipStream_t st) {
#define HYLRA_G(GG)                                                          \
    if (G == GG) {                                                           \
        if (D == 128) return launch_g<128, GG>(p, B, NB, nt, NW, st);        \
        if (D == 64) return launch_g<64, GG>(p, B, NB, nt, NW, st);          \
    }
    HYLRA_G(1) HYLRA_G(2) HYLRA_G(3) HYLRA_G(4) HYLRA_G(5) HYLRA_G(6) HYLRA_G(7) HYLRA_G(8)
#undef HYLRA_G
    return hipErrorInvalidValue;
}

}  // namespace hylra
