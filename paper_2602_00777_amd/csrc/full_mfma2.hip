// Full layer, streaming pass (Algorithm 2, Full branch) for head_dim 128 with a wave's work in
// the second matrix-core form (mfma2_core.h): whole-line K loads by lane pairs, whole-row V
// loads transposed inside the lane, both contractions of Eq. 1 on v_mfma_f32_16x16x32_bf16.
// Same role, outputs and launch geometry as the vector kernel (full_attn_impl.h) and the first
// matrix-core kernel (full_mfma.hip): per-head online-softmax partials, the group-mean score of
// every row, their range per split.  Loop shape as in the vector kernel's pipelined mode: a
// wave tile is 32 rows, the loads of tile i+1 are issued (unconditionally, rows clamped to the
// split's last row) before tile i is consumed, and the scores are staged in LDS and written
// once after the loop, so that no vector store sits between the loads.  DYN: the rows are
// handed out at run time (chunk_queue.h) instead of split evenly; scores are then staged by
// ticket as in the vector kernel.
#include "chunk_queue.h"
#include "launch.h"
#include "mfma2_core.h"
#include "score_hist.h"

namespace hylra {

struct Tile32 {
    uint4 k[2][4];      // blocks a, b: the lane-pair loads of K (see own_row)
    uint4 v[8];         // rows 4 gq + j of a (j < 4) and of b (j >= 4), columns 8 n ..
};

template <int G, bool DYN>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void full_mfma2_kernel(FullParams p) {
    constexpr int D = 128, NW = 4, TILE = 32, STEP = NW * TILE;
    __shared__ float s_m[NW][16];
    __shared__ float s_l[NW][16];
    __shared__ __attribute__((aligned(16))) float s_acc[NW * G * D];
    __shared__ int s_hist[kScoreBins];
    extern __shared__ float s_scores[];          // [rows_per_split], then the staged page table

    int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    int my_wgs = p.wgs_per_seg;                              // workgroups of this pair (DYN)
    int64_t slot0 = ((int64_t)b * p.Hkv + g) * p.n_splits;   // the pair's first partial slot
    int mapped_rows = -1;
    if (DYN && !p.wg_map && p.gen_half) {
        // early and late arrivals on the compute units are mixed in every group of workgroups
        int unit, w;
        paired_unit((int)(blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z)), p.gen_half, p.wgs_per_seg,
                    unit, w);
        const int pair = unit / p.n_segs;
        b = pair / p.Hkv, g = pair - b * p.Hkv;
        split = (unit - pair * p.n_segs) * p.wgs_per_seg + w;
        slot0 = (int64_t)pair * p.n_splits;
    }
    if (DYN && p.wg_map) {
        // sequences of different lengths: the pairs' shares of the workgroups were dealt out before the launch
        const int4 m = p.wg_map[slot0 + split];
        if ((m.y >> 16) == 0) return;
        b = m.x / p.Hkv, g = m.x - b * p.Hkv;
        split = m.y & 0xffff, my_wgs = m.y >> 16, slot0 = m.z, mapped_rows = m.w;
    }
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, gq = lane >> 4;

    const bool paged = p.map.table != nullptr;
    const int64_t base = (paged ? 0 : (int64_t)b * p.sb) + (int64_t)g * p.sh;
    const uint16_t* __restrict__ Kb = p.K + base;
    const uint16_t* __restrict__ Vb = p.V + base;
    const int64_t head0 = (int64_t)b * p.Hq + (int64_t)g * G;
    HYLRA_TS(0);
    uint4 qb[4];
    mfma_load_q<D, G>(qb, p.q + head0 * D, n, gq);
    State2 st;
    st.init();

    // rows of this sequence; a shorter sequence is cut into the same number of (shorter) splits
    const int n_rows = mapped_rows >= 0 ? mapped_rows : seq_rows(p.map, b, p.N);
    const int rps = DYN || n_rows == p.N ? p.rows_per_split
                                         : (n_rows + p.n_splits * STEP - 1) / (p.n_splits * STEP) * STEP;
    const int row0 = DYN ? 0 : split * rps;
    const int row1 = DYN ? n_rows : min(n_rows, row0 + rps);
    // p.scores == nullptr: nobody will rank this layer's rows (its index set is not wanted), so
    // the group-mean scores are neither formed nor written, nor is their range
    const bool want_scores = p.scores != nullptr;
    float* __restrict__ srow = want_scores ? p.scores + ((int64_t)b * p.Hkv + g) * p.score_stride : nullptr;
    // the scores are also counted, as they are formed, per top 12 bits of their key
    // (score_hist.h)
    const bool bins = want_scores && p.ghist != nullptr;
    if (bins) hist_zero<NW * 64>(s_hist);
    if (!DYN && bins) __syncthreads();           // (the other form meets at a barrier before its first tile anyway)

    // paged cache: the split's part of the sequence's page table, staged in LDS (read from
    // memory if it does not fit there)
    int* const s_tbl = reinterpret_cast<int*>(s_scores + p.rows_per_split);
    int* const s_tile_of = s_tbl + p.tbl_cap;    // DYN: the tile whose scores staging slot t (= ticket t) holds
    const int32_t* __restrict__ tbl = p.map.table + (int64_t)b * p.map.table_stride;     // unused unless paged
    int tbl_page0 = -1;
    auto stage_table = [&](int first_row, int last_row) {                   // every thread; rows of this sequence
        const int page0 = first_row >> p.map.page_shift, n_pages = (last_row >> p.map.page_shift) - page0 + 1;
        if (n_pages <= p.tbl_cap) {
            for (int i = tid; i < n_pages; i += NW * 64) s_tbl[i] = tbl[page0 + i];
            tbl_page0 = page0;
        }
        __syncthreads();
    };
    if (!DYN && paged && row0 < row1) stage_table(row0, row1 - 1);
    auto row_offset = [&](int row) -> int64_t {
        if (!paged) return (int64_t)row * p.sn;
        const int t = row >> p.map.page_shift;
        const int page = tbl_page0 >= 0 ? s_tbl[t - tbl_page0] : tbl[t];
        return (int64_t)page * p.map.stride_page + (int64_t)(row & ((1 << p.map.page_shift) - 1)) * p.sn;
    };

    // Rows past `last` (the split's last row by default) are clamped to it and masked later.
    // A block of 16 rows starts at a multiple of 16, so with pages of 16 rows or more it lies
    // inside one page (as it trivially does in a contiguous cache): one 64-bit offset per block
    // (one page-table lookup) and 32-bit distances from it for the lanes' rows.  Smaller pages:
    // every row is looked up (also with row strides so large that 16 of them overflow 32 bits).
    const bool by_block = (!paged || p.map.page_shift >= 4) && p.sn < (1 << 26);
    const int sn = (int)p.sn;
    auto issue = [&](Tile32& buf, int t0, int last = -1) {
        if (last < 0) last = row1 - 1;
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
            const int r0 = t0 + 16 * blk;
            const int ra = min(r0 + (n & 7), last), rb = min(r0 + 8 + (n & 7), last);
            int64_t offa, offb, offv[4];
            if (by_block) {
                const int rc = min(r0, last);                    // <= every clamped row of the block
                const int64_t blk_base = row_offset(rc);
                offa = blk_base + (ra - rc) * sn;
                offb = blk_base + (rb - rc) * sn;
#pragma unroll
                for (int j = 0; j < 4; ++j) offv[j] = blk_base + (min(r0 + 4 * gq + j, last) - rc) * sn;
            } else {
                offa = row_offset(ra);
                offb = row_offset(rb);
#pragma unroll
                for (int j = 0; j < 4; ++j) offv[j] = row_offset(min(r0 + 4 * gq + j, last));
            }
            offa += 32 * (n >> 3) + 8 * gq;
            offb += 32 * (n >> 3) + 8 * gq;
#pragma unroll
            for (int L = 0; L < 2; ++L) {
                buf.k[blk][2 * L] = ld16<true>(Kb + offa + 64 * L);
                buf.k[blk][2 * L + 1] = ld16<true>(Kb + offb + 64 * L);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) buf.v[4 * blk + j] = ld16<true>(Vb + offv[j] + 8 * n);
        }
    };
    // st0: where the tile's scores are staged in s_scores (negative: store to memory)
    auto consume = [&](Tile32& buf, int t0, int st0) {
        own_row(buf.k[0]);
        own_row(buf.k[1]);
        const int left = row1 - t0;                          // rows of this tile inside the split
        const uint32_t mask_a = left >= 16 ? 0xffffu : left > 0 ? (1u << left) - 1u : 0u;
        const uint32_t mask_b = left >= 32 ? 0xffffu : left > 16 ? (1u << (left - 16)) - 1u : 0u;
        float4_t Sa, Sb;
        group32<G>(st, buf.k[0], buf.k[1], buf.v, qb, mask_a, mask_b, p.scale_log2, n, gq, Sa, Sb);
        if (!want_scores) return;
        // group-mean score of rows 4 gq + j of each block: sum over the 16 head lanes (padding
        // heads hold 0), which leaves every lane of a 16-lane row with the row's eight values.
        // Lane n < 8 keeps value n (block n >> 2, row 4 gq + (n & 3) of it): one LDS store and one
        // histogram count per tile for 32 lanes.  Staged in LDS at the row's place in the split.
        float mine = 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            float v = group_sum<16>((c >> 2) ? Sb[c & 3] : Sa[c & 3]) * p.scale_mean;
            v = fminf(fmaxf(v, -3.0e38f), 3.0e38f);          // also maps NaN to a number
            mine = n == c ? v : mine;
        }
        const int r = 16 * (n >> 2) + 4 * gq + (n & 3);
        if (n < 8 && r < left) {
            if (DYN && st0 < 0) srow[t0 + r] = mine;
            else s_scores[st0 + r] = mine;
            if (bins) hist_add(s_hist, mine);
        }
    };

    if (DYN && n_rows > 0) {
        __shared__ ChunkQueue cq;
        const int tiles_b = (n_rows + TILE - 1) / TILE;            // tiles of this sequence
        SegInfo sg;
        sg.made_for = p.made_for;
        int w;
        int* ctr;
        if (mapped_rows >= 0) {
            // the pair's own number of workgroups, in segments of their own (counters: the pair's partial slots)
            const PairSeg ps = pair_segment(my_wgs, p.wgs_per_seg, split);
            w = ps.w;
            sg.wgs = ps.wgs;
            sg.tile0 = (int)((int64_t)tiles_b * ps.wg0 / my_wgs);
            sg.tiles = (int)((int64_t)tiles_b * (ps.wg0 + ps.wgs) / my_wgs) - sg.tile0;
            ctr = p.chunk_ctr + (slot0 + ps.seg) * kCtrStride;
        } else {
            const int seg = split / my_wgs;
            w = split - seg * my_wgs;
            sg.wgs = my_wgs;
            sg.tile0 = 0, sg.tiles = tiles_b;
            if (p.n_segs > 1) {             // (the 64-bit divisions are left out of the common case)
                sg.tile0 = (int)((int64_t)seg * tiles_b / p.n_segs);
                sg.tiles = (int)((int64_t)(seg + 1) * tiles_b / p.n_segs) - sg.tile0;
            }
            ctr = p.chunk_ctr + (((int64_t)b * p.Hkv + g) * p.n_segs + seg) * kCtrStride;
        }
        seg_chunks(p, sg);
        // a row of the segment that exists: where a wave with nothing left points its loads
        // (all of them at this one row: the rows after it may lie outside the staged table)
        const int idle_row = min(sg.tile0 * TILE, n_rows - 1);
        if (paged) stage_table(idle_row, max(idle_row, min((sg.tile0 + sg.tiles) * TILE, n_rows) - 1));
        // The chunk the workgroup starts on is known without the queue: wave v takes its tile v
        // and has the loads under way while thread 0 sets the queue up (the draw of a chunk's
        // first tile also claims the workgroup's next chunk: wave 0 does that first, so that the
        // claim's answer is not queued behind the tile).
        int lo0 = 0, hi0 = 0;
        if (w < sg.n_eff) lo0 = chunk_bound(p, sg, w), hi0 = chunk_bound(p, sg, w + 1);
        const bool early = wave < hi0 - lo0;
        PendingClaim pc;
        pc.raw = 0, pc.slot = -1, pc.first = 0;
        Tile32 bufA, bufB;
        TileRef ta;
        ta.tile = -1, ta.ticket = wave;
        if (early) {
            if (wave == 0) {
                if (lane == 0) pc.raw = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                pc.slot = 1, pc.first = hi0 - lo0;
            }
            ta.tile = sg.tile0 + lo0 + wave;
            issue(bufA, ta.tile * TILE);
        }
        if (tid == 0) {
            int lo = lo0, hi = hi0;
            bool has = hi0 > lo0;
            if (w < sg.n_eff && !has) {
                const int raw = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                has = settle_claim(p, sg, ctr, raw, lo, hi) >= 0;
            }
            cq.ticket = min(max(hi0 - lo0, 0), NW);          // the tiles taken above
            cq.first[0] = 0;
            cq.first[1] = has ? hi - lo : 0;
            cq.tile0[0] = has ? sg.tile0 + lo : 0;
            cq.n_ready = 1;
            cq.done = has ? 0 : 1;
            cq.gave_up = 0;
        }
        __syncthreads();
        QueueCursor cur;
        cur.slot = 0;
        cur.first = 0;
        cur.next = lds_load(&cq.first[1]);
        cur.tile0 = lds_load(&cq.tile0[0]);
        const int stage_tiles = p.rows_per_split / TILE;      // tiles the staging area holds
        auto stage_of = [&](const TileRef& t) {
            if (t.ticket >= stage_tiles) return -1;
            if (lane == 0) s_tile_of[t.ticket] = t.tile;
            return t.ticket * TILE;
        };
        if (!early) {
            ta = next_tile(cq, ctr, cur, pc, lane);
            issue(bufA, ta.tile >= 0 ? ta.tile * TILE : idle_row, ta.tile >= 0 ? -1 : idle_row);
        }
        HYLRA_TS(5);
        while (ta.tile >= 0) {
            publish_claim(cq, p, ctr, pc, lane, sg);                  // (first pass only)
            const TileRef tb = next_tile(cq, ctr, cur, pc, lane);
            issue(bufB, tb.tile >= 0 ? tb.tile * TILE : idle_row, tb.tile >= 0 ? -1 : idle_row);    // nothing left: a harmless reload
            consume(bufA, ta.tile * TILE, stage_of(ta));
            publish_claim(cq, p, ctr, pc, lane, sg);
            if (tb.tile < 0) break;
            ta = next_tile(cq, ctr, cur, pc, lane);
            issue(bufA, ta.tile >= 0 ? ta.tile * TILE : idle_row, ta.tile >= 0 ? -1 : idle_row);
            consume(bufB, tb.tile * TILE, stage_of(tb));
            publish_claim(cq, p, ctr, pc, lane, sg);
        }
        publish_claim(cq, p, ctr, pc, lane, sg);
        HYLRA_TS(1);
        __syncthreads();
        report_give_up(cq, p.err_word);
        HYLRA_TS(2);
        // write the staged scores out: 8 threads per staged tile, 16 bytes each (tile starts and
        // the score stride are multiples of 4 floats, so the stores are aligned)
        const int n_staged = want_scores ? min(cq.first[cq.n_ready], stage_tiles) : 0;
        for (int i = tid; i < n_staged * (TILE / 4); i += NW * 64) {
            const int t = i >> 3, part = i & 7;
            const int r = s_tile_of[t] * TILE + 4 * part;
            const float* src = s_scores + t * TILE + 4 * part;
            if (r + 4 <= n_rows) {
                *reinterpret_cast<float4*>(srow + r) = *reinterpret_cast<const float4*>(src);
            } else {
                for (int x = 0; x < 4; ++x)
                    if (r + x < n_rows) srow[r + x] = src[x];
            }
        }
    } else if (!DYN && row0 < row1) {
        Tile32 bufA, bufB;
        int t0 = row0 + wave * TILE;
        issue(bufA, t0);
        while (t0 < row1) {
            issue(bufB, t0 + STEP);
            consume(bufA, t0, t0 - row0);
            t0 += STEP;
            if (t0 >= row1) break;
            issue(bufA, t0 + STEP);
            consume(bufB, t0, t0 - row0);
            t0 += STEP;
        }
    }

    HYLRA_TS(3);
    if (!DYN) {
        __syncthreads();                         // every score of the split is in LDS
        // row0 and the score stride are multiples of 4 floats: 16-byte stores are aligned
        float* __restrict__ dst = srow + row0;
        const int cnt = want_scores ? max(row1 - row0, 0) : 0;
        for (int i = 4 * tid; i < cnt; i += 4 * NW * 64) {
            if (i + 4 <= cnt) {
                *reinterpret_cast<float4*>(dst + i) = *reinterpret_cast<const float4*>(s_scores + i);
            } else {
                for (int e = i; e < cnt; ++e) dst[e] = s_scores[e];
            }
        }
    }
    // the pair's partials: [head of the group][partial] from slot0 * G on
    const int n_part = DYN ? my_wgs * p.n_segs : p.n_splits;
    merge_store2<G, NW, false>(st, s_m, s_l, s_acc, p.part_ml + (slot0 * G + split) * 2,
                               (int64_t)n_part * 2, p.part_acc + (slot0 * G + split) * D,
                               (int64_t)n_part * D, n, gq);
    // (the barrier inside the merge lies between the last count and the flush)
    if (bins) hist_flush<NW * 64>(s_hist, p.ghist + ((int64_t)b * p.Hkv + g) * kScoreBins);
    HYLRA_TS(4);
}

// rows a workgroup consumes per sweep of its 4 waves; variant 72 = even splits, 74 = rows handed
// out at run time
int full_mfma2_quantum(int D, int variant) { return (D == 128 && (variant == 72 || variant == 74)) ? 128 : 0; }

hipError_t launch_full_mfma2(const FullParams& p, int B, int G, int variant, hipStream_t st) {
    if (variant != 72 && variant != 74) return hipErrorInvalidValue;
    dim3 grid(p.n_splits, p.Hkv, B);
    // scores of the split (or staging area), staged page table, and (variant 74) a tile number per staged tile
    const size_t lds = p.rows_per_split * sizeof(float) + p.tbl_cap * sizeof(int) +
                       (variant == 74 ? p.rows_per_split / 32 * sizeof(int) : 0);
#define HYLRA_G(GG)                                                                                   \
    if (G == GG) {                                                                                    \
        if (variant == 74) hipLaunchKernelGGL((full_mfma2_kernel<GG, true>), grid, dim3(256), lds, st, p);  \
        else hipLaunchKernelGGL((full_mfma2_kernel<GG, false>), grid, dim3(256), lds, st, p);         \
        return hipGetLastError();                                                                     \
    }
    HYLRA_G(1) HYLRA_G(2) HYLRA_G(3) HYLRA_G(4) HYLRA_G(5) HYLRA_G(6) HYLRA_G(7) HYLRA_G(8)
#undef HYLRA_G
    return hipErrorInvalidValue;
}

}  // namespace hylra
