// Reuse layer (Algorithm 2, Reuse branch; attention as in Eq. 1) for head_dim 128, second
// matrix-core form: same decomposition and cross-workgroup merge as reuse_mfma.hip; how the
// rows are fetched and contracted is described in mfma2_core.h.
#include "launch.h"
#include "mfma2_core.h"
#include "reuse_tail.h"

namespace hylra {

// A wave takes NB blocks of 16 index entries (= NB / 2 groups of 32) per sweep; NW waves per
// workgroup.
template <int G, bool NT, int NW, int NB>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2))) void reuse_mfma2_kernel(ReuseParams p) {
    constexpr int D = 128, ROWS_W = 16 * NB;
    __shared__ float s_m[NW][16];
    __shared__ float s_l[NW][16];
    __shared__ __attribute__((aligned(16))) float s_acc[NW * G * D];
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

    const int page_mask = (1 << p.map.page_shift) - 1;
    // element offset of a row given its place (see below)
    auto place = [&](int pr) -> int64_t {
        return tbl ? (int64_t)(pr >> p.map.page_shift) * p.map.stride_page + (int64_t)(pr & page_mask) * p.sn
                   : (int64_t)pr * p.sn;
    };
    // a negative place stands for the token being appended, whose rows are not in the cache yet
    auto k_at = [&](int pr) -> const uint16_t* { return pr < 0 ? nr.k : Kb + place(pr); };
    auto v_at = [&](int pr) -> const uint16_t* { return pr < 0 ? nr.v : Vb + place(pr); };
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
    uint4 qb[4];
    mfma_load_q<D, G>(qb, p.q + head0 * D, n, gq);
    State2 st;
    st.init();

    while (t0 < i1) {
        HYLRA_TS(1);
        uint4 kb[NB][4], vb[NB][4];
        bool valid[NB];
#pragma unroll
        for (int blk = 0; blk < NB; ++blk) {
            valid[blk] = (unsigned)row[blk] < (unsigned)n_rows;    // negative or past the sequence: padding
            // Where the lane's row lives: its number in a contiguous cache, page * page_size +
            // slot in a paged one (one page-table lookup per row; the lanes below that fetch
            // pieces of other lanes' rows get this number from them, not from the table).
            const int r = valid[blk] ? row[blk] : 0;
            const int pr = r == nr.row ? -1 : tbl ? (tbl[r >> p.map.page_shift] << p.map.page_shift) | (r & page_mask) : r;
            // K: lanes n and n ^ 8 read the two halves of a 128-byte line of one row (row n & 7
            // of the block in the first load of a line, row 8 + (n & 7) in the second), so that
            // eight lanes cover a whole line; own_row() afterwards hands every lane the pieces of
            // its own row n.
            const int ra = rotate_in<0xC>(pr, pr);                  // lanes 8..15: from lane n - 8
            const int rb = rotate_in<0x3>(pr, pr);                  // lanes 0..7: from lane n + 8
            const uint16_t* pa = k_at(ra) + 32 * (n >> 3) + 8 * gq;
            const uint16_t* pb = k_at(rb) + 32 * (n >> 3) + 8 * gq;
#pragma unroll
            for (int L = 0; L < 2; ++L) {
                kb[blk][2 * L] = ld16<NT>(pa + 64 * L);
                kb[blk][2 * L + 1] = ld16<NT>(pb + 64 * L);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // row 4 gq + j of the block: its place sits in lane 4 gq + j
                const int rv = __shfl(pr, 4 * gq + j, 64);
                vb[blk][j] = ld16<NT>(v_at(rv) + 8 * n);
            }
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
        for (int gp = 0; gp < NB / 2; ++gp) {
            // lanes 0..15 carry the 16 rows' validity
            const uint32_t mask_a = (uint32_t)__builtin_amdgcn_ballot_w64(valid[2 * gp]) & 0xffffu;
            const uint32_t mask_b = (uint32_t)__builtin_amdgcn_ballot_w64(valid[2 * gp + 1]) & 0xffffu;
            uint4 v8[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v8[j] = vb[2 * gp][j];
                v8[4 + j] = vb[2 * gp + 1][j];
            }
            own_row(kb[2 * gp]);
            own_row(kb[2 * gp + 1]);
            float4_t Sa, Sb;
            group32<G>(st, kb[2 * gp], kb[2 * gp + 1], v8, qb, mask_a, mask_b, p.scale_log2, n, gq, Sa, Sb);
        }
        HYLRA_TS(2);
    }

    float* const my_ml = p.part_ml + (head0 * p.n_splits + split) * 2;
    float* const my_acc = p.part_acc + (head0 * p.n_splits + split) * D;
    const int64_t ml_stride = (int64_t)p.n_splits * 2, acc_stride = (int64_t)p.n_splits * D;
    if (p.n_splits == 1 && p.counters) {    // nothing crosses workgroups: no partial, no counter
        stage_states2<G, NW>(st, s_m, s_l, s_acc, n, gq);
        staged_to_output<D, G, NW>(s_m, s_l, s_acc, p.out + head0 * D);
        return;
    }
    if (p.packets) {                        // every workgroup merges its slice of the columns
        __shared__ float s_pk[kPacketUnitsPerThread * NW * 64];
        HYLRA_TS(3);
        stage_states2<G, NW>(st, s_m, s_l, s_acc, n, gq);
        uint64_t* pk_pair = p.packets + pair * p.n_splits * p.n_splits * packet_shape(G, D, p.n_splits).PK;
        send_packets<G, D, NW * 64>(
            pk_pair, p.n_splits, split, [&](int h) { return staged_max<NW>(s_m, h); },
            [&](int h, float M) { return staged_sum<NW>(s_m, s_l, h, M); },
            [&](int h, int col, float M) { return staged_acc<G, NW>(s_m, s_acc, h, col, M); });
        reuse_packet_tail<G, D, NW * 64>(p, pk_pair, head0, split, s_pk);
        return;
    }
    if (p.counters == nullptr) {            // unfused: a separate kernel merges the partials
        merge_store2<G, NW, false>(st, s_m, s_l, s_acc, my_ml, ml_stride, my_acc, acc_stride, n, gq);
        return;
    }
    merge_store2<G, NW, true>(st, s_m, s_l, s_acc, my_ml, ml_stride, my_acc, acc_stride, n, gq);
    reuse_merge_tail<G, D, NW * 64>(p, pair, head0, &s_last);
}

template <int G>
static hipError_t launch2_g(const ReuseParams& p, int B, bool nt, int NW, int NB, hipStream_t st) {
    dim3 grid(p.n_splits, p.Hkv, B);
#define HYLRA_CASE(NWV, NBV)                                                                              \
    if (NW == NWV && NB == NBV) {                                                                         \
        if (nt) hipLaunchKernelGGL((reuse_mfma2_kernel<G, true, NWV, NBV>), grid, dim3(NWV * 64), 0, st, p); \
        else hipLaunchKernelGGL((reuse_mfma2_kernel<G, false, NWV, NBV>), grid, dim3(NWV * 64), 0, st, p);   \
        return hipGetLastError();                                                                         \
    }
    HYLRA_CASE(4, 4)
    HYLRA_CASE(8, 4)
    HYLRA_CASE(4, 2)
#undef HYLRA_CASE
    return hipErrorInvalidValue;
}

// index entries per workgroup sweep (NW waves of NB blocks of 16); 0 if the shape is not built
int reuse_mfma2_quantum(int D, int NW, int NB) {
    return (D == 128 && ((NB == 4 && (NW == 4 || NW == 8)) || (NB == 2 && NW == 4))) ? NW * NB * 16 : 0;
}

hipError_t launch_reuse_mfma2(const ReuseParams& p, int B, int G, bool nt, int NW, int NB, hipStream_t st) {
#define HYLRA_G(GG) \
    if (G == GG) return launch2_g<GG>(p, B, nt, NW, NB, st);
    HYLRA_G(1) HYLRA_G(2) HYLRA_G(3) HYLRA_G(4) HYLRA_G(5) HYLRA_G(6) HYLRA_G(7) HYLRA_G(8)
#undef HYLRA_G
    return hipErrorInvalidValue;
}

}  // namespace hylra
