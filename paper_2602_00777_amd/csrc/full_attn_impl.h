// Full layer, streaming pass (Algorithm 2, Full branch): one split of the KV rows of one
// (batch, KV head) per workgroup.  Reads every K and V row of the split exactly once,
// produces per-head online-softmax partials, and the group-mean scaled score of every row
// (the quantity TopK ranks) for the finalise kernel.
#pragma once
#include "attend.h"
#include "chunk_queue.h"
#include "launch.h"
#include "score_hist.h"

#ifndef HYLRA_BUILD_D
#error "define HYLRA_BUILD_D to 64 or 128"
#endif

namespace hylra {

// MODE 2: streaming (non-temporal) loads and a two-deep register pipeline -- the loads of tile
// i+1 are issued before tile i is consumed, so every wave always has one to two tiles in flight.
//
// The group-mean scores of the split are staged in LDS (rows_per_split floats of dynamic
// shared memory) and written out once, after the loop.  Besides turning them into full
// 16-byte stores this keeps vector stores out of the loop: loads and stores share one
// completion counter on this architecture and do not complete in order with respect to each
// other, so with a store pending every wait for a tile would have to drain the counter to
// zero, i.e. also wait for the tile that was only just requested.  For the same reason the
// pipelined loop issues its look-ahead loads unconditionally (rows past the split are
// clamped to its last row): the number of younger loads at each wait is then a constant.
// MODE 4: as MODE 2, but the rows are handed out at run time (chunk_queue.h).  Group-mean
// scores are staged in LDS by ticket (the workgroup's t-th tile at t * TILE) and written out
// after the loop, slot by slot.  (A store inside the loop, even once per chunk, costs more
// than it saves: loads and stores share one completion counter and complete out of order with
// respect to each other, so every store means draining the wave's loads once.)  Tickets
// beyond the staging area (a workgroup that ends up with far more than its share) store
// straight to memory.
template <int D, int G, int CH, int R, int MODE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void full_attn_split_kernel(FullParams p) {
    using GEO = Geo<D, G, CH>;
    constexpr int NW = 4;
    constexpr int TILE = R * GEO::RPG;
    constexpr bool NT = true;
    __shared__ float smem[merge_smem_floats<GEO, NW>()];
    __shared__ int s_hist[kScoreBins];
    extern __shared__ float s_scores[];          // [rows_per_split]

    int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    int my_wgs = p.wgs_per_seg;                              // workgroups of this pair (self-scheduling mode)
    int64_t slot0 = ((int64_t)b * p.Hkv + g) * p.n_splits;   // the pair's first partial slot
    int mapped_rows = -1;
    if (MODE == 4 && !p.wg_map && p.gen_half) {
        // early and late arrivals on the compute units are mixed in every group of workgroups
        int unit, w;
        paired_unit((int)(blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z)), p.gen_half, p.wgs_per_seg,
                    unit, w);
        const int pair = unit / p.n_segs;
        b = pair / p.Hkv, g = pair - b * p.Hkv;
        split = (unit - pair * p.n_segs) * p.wgs_per_seg + w;
        slot0 = (int64_t)pair * p.n_splits;
    }
    if (MODE == 4 && p.wg_map) {
        // sequences of different lengths: the pairs' shares of the workgroups were dealt out before the launch
        const int4 m = p.wg_map[slot0 + split];
        if ((m.y >> 16) == 0) return;
        b = m.x / p.Hkv, g = m.x - b * p.Hkv;
        split = m.y & 0xffff, my_wgs = m.y >> 16, slot0 = m.z, mapped_rows = m.w;
    }
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunk = lane % GEO::LPR, slot = lane / GEO::LPR;

    HYLRA_TS(0);
    const bool paged = p.map.table != nullptr;
    const int64_t base = (paged ? 0 : (int64_t)b * p.sb) + (int64_t)g * p.sh;
    const uint16_t* __restrict__ Kb = p.K + base;
    const uint16_t* __restrict__ Vb = p.V + base;
    uint4 qv[G][CH];
    load_q<GEO>(qv, p.q + ((int64_t)b * p.Hq + (int64_t)g * G) * D, chunk);

    LaneState<GEO> st;
    st.init();
    constexpr bool DYN = MODE == 4;
    constexpr int STEP = NW * TILE;
    // rows of this sequence; a shorter sequence is cut into the same number of (shorter) splits
    const int n_rows = mapped_rows >= 0 ? mapped_rows : seq_rows(p.map, b, p.N);
    const int rps = DYN || n_rows == p.N ? p.rows_per_split
                                         : (n_rows + p.n_splits * STEP - 1) / (p.n_splits * STEP) * STEP;
    const int row0 = DYN ? 0 : split * rps;
    const int row1 = DYN ? n_rows : min(n_rows, row0 + rps);
    float* __restrict__ srow = p.scores + ((int64_t)b * p.Hkv + g) * p.score_stride;
    // the scores are also counted per top 12 bits of their key (score_hist.h); a barrier follows
    // on every path before the first count
    const bool bins = p.ghist != nullptr;
    if (bins) hist_zero<NW * 64>(s_hist);

    // Paged cache: the part of the sequence's page table this workgroup can touch is staged in
    // LDS behind the score staging area (a lookup from memory in the loop would put a load
    // between the tiles' loads, whose result the address arithmetic would have to wait for).
    // If it does not fit there (tiny pages, long contexts) the table is read from memory.
    int* const s_tbl = reinterpret_cast<int*>(s_scores + p.rows_per_split);
    const int32_t* __restrict__ tbl = p.map.table + (int64_t)b * p.map.table_stride;     // unused unless paged
    int tbl_page0 = -1;                                                     // first staged page; -1: not staged
    auto stage_table = [&](int first_row, int last_row) {                   // every thread; rows of this sequence
        const int page0 = first_row >> p.map.page_shift, n_pages = (last_row >> p.map.page_shift) - page0 + 1;
        if (n_pages <= p.tbl_cap) {
            for (int i = tid; i < n_pages; i += NW * 64) s_tbl[i] = tbl[page0 + i];
            tbl_page0 = page0;
        }
        __syncthreads();
    };
    auto row_offset = [&](int row) -> int64_t {
        if (!paged) return (int64_t)row * p.sn;
        const int t = row >> p.map.page_shift;
        const int page = tbl_page0 >= 0 ? s_tbl[t - tbl_page0] : tbl[t];
        return (int64_t)page * p.map.stride_page + (int64_t)(row & ((1 << p.map.page_shift) - 1)) * p.sn;
    };

    // element offsets of this lane's rows in the tile starting at row t0; rows past `last`
    // (the split's last row by default) are clamped to it and masked when consumed
    auto offsets = [&](int t0, int64_t (&off)[R], int last = -1) {
        if (last < 0) last = row1 - 1;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int row = min(t0 + r * GEO::RPG + slot, last);
            off[r] = row_offset(row) + chunk * 8;
        }
    };
    // softmax/accumulate a loaded tile, stage its group-mean scores, track their range
    // st0: where the tile's scores are staged in s_scores (static modes: t0 - row0; dynamic:
    // ticket * TILE, or negative = store to memory)
    auto consume = [&](const TileBuf<GEO, R>& buf, int t0, int st0) {
        bool valid[R];
        float ms[R];
        if (t0 + TILE <= row1) {
#pragma unroll
            for (int r = 0; r < R; ++r) valid[r] = true;
            compute_tile<GEO, R, false>(st, qv, buf, valid, p.scale_log2, p.scale_mean, ms);
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const float v = fminf(fmaxf(ms[r], -3.0e38f), 3.0e38f);   // also maps NaN to a number
                if (chunk == 0) {
                    if (DYN && st0 < 0) {
                        srow[t0 + r * GEO::RPG + slot] = v;
                        if (bins) hist_add(s_hist, v);
                    } else {
                        s_scores[st0 + r * GEO::RPG + slot] = v;
                    }
                }
            }
        } else {
#pragma unroll
            for (int r = 0; r < R; ++r) valid[r] = t0 + r * GEO::RPG + slot < row1;
            compute_tile<GEO, R, true>(st, qv, buf, valid, p.scale_log2, p.scale_mean, ms);
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const float v = fminf(fmaxf(ms[r], -3.0e38f), 3.0e38f);
                if (valid[r] && chunk == 0) {
                    if (DYN && st0 < 0) {
                        srow[t0 + r * GEO::RPG + slot] = v;
                        if (bins) hist_add(s_hist, v);
                    } else {
                        s_scores[st0 + r * GEO::RPG + slot] = v;
                    }
                }
            }
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
        if (tid == 0) {
            int lo = 0, hi = 0;
            bool has = false;
            if (w < sg.n_eff) {
                lo = chunk_bound(p, sg, w);
                hi = chunk_bound(p, sg, w + 1);
                has = hi > lo;
                if (!has) {
                    const int raw = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    has = settle_claim(p, sg, ctr, raw, lo, hi) >= 0;
                }
            }
            cq.ticket = 0;
            cq.first[0] = 0;
            cq.first[1] = has ? hi - lo : 0;
            cq.tile0[0] = has ? sg.tile0 + lo : 0;
            cq.n_ready = 1;
            cq.done = has ? 0 : 1;
            cq.gave_up = 0;
        }
        __syncthreads();
        QueueCursor qslot;
        qslot.slot = 0;
        qslot.first = 0;
        qslot.next = lds_load(&cq.first[1]);
        qslot.tile0 = lds_load(&cq.tile0[0]);
        TileBuf<GEO, R> bufA, bufB;
        int64_t off[R];
        const int stage_tiles = p.rows_per_split / TILE;      // tiles the staging area holds
        auto stage_of = [&](const TileRef& t) { return t.ticket < stage_tiles ? t.ticket * TILE : -1; };
        PendingClaim pc;
        pc.raw = 0, pc.slot = -1, pc.first = 0;
        TileRef ta = next_tile(cq, ctr, qslot, pc, lane);
        offsets(ta.tile >= 0 ? ta.tile * TILE : idle_row, off, ta.tile >= 0 ? -1 : idle_row);
        load_tile<GEO, R, NT>(bufA, Kb, Vb, off);
        while (ta.tile >= 0) {
            publish_claim(cq, p, ctr, pc, lane, sg);                      // (first pass only)
            const TileRef tb = next_tile(cq, ctr, qslot, pc, lane);
            offsets(tb.tile >= 0 ? tb.tile * TILE : idle_row, off, tb.tile >= 0 ? -1 : idle_row);   // nothing left: a harmless reload
            load_tile<GEO, R, NT>(bufB, Kb, Vb, off);
            consume(bufA, ta.tile * TILE, stage_of(ta));
            publish_claim(cq, p, ctr, pc, lane, sg);
            if (tb.tile < 0) break;
            ta = next_tile(cq, ctr, qslot, pc, lane);
            offsets(ta.tile >= 0 ? ta.tile * TILE : idle_row, off, ta.tile >= 0 ? -1 : idle_row);
            load_tile<GEO, R, NT>(bufA, Kb, Vb, off);
            consume(bufB, tb.tile * TILE, stage_of(tb));
            publish_claim(cq, p, ctr, pc, lane, sg);
        }
        publish_claim(cq, p, ctr, pc, lane, sg);
        __syncthreads();
        report_give_up(cq, p.err_word);
        // write the staged scores out: slot i of the queue is tiles tile0[i] .. of the pair,
        // tickets first[i] .. first[i + 1] - 1 (tile starts and the score stride are multiples
        // of 4 floats, so the 16-byte stores are aligned)
        const int n_slots = cq.n_ready;
        for (int i = 0; i < n_slots; ++i) {
            const int f0 = cq.first[i], f1 = min(cq.first[i + 1], stage_tiles);
            const int r0 = cq.tile0[i] * TILE;
            const int n = min((f1 - f0) * TILE, n_rows - r0);
            const float* src = s_scores + f0 * TILE;
            for (int e = 4 * tid; e < n; e += 4 * NW * 64) {
                if (e + 4 <= n) {
                    *reinterpret_cast<float4*>(srow + r0 + e) = *reinterpret_cast<const float4*>(src + e);
                } else {
                    for (int x = e; x < n; ++x) srow[r0 + x] = src[x];
                }
                if (bins)
                    for (int x = e; x < min(e + 4, n); ++x) hist_add(s_hist, src[x]);
            }
        }
    } else if (DYN || row0 >= row1) {
        // nothing to stream: an empty sequence, or a split past the end of a short one
    } else {
        if (paged) stage_table(row0, row1 - 1);
        TileBuf<GEO, R> bufA, bufB;
        int64_t off[R];
        int t0 = row0 + wave * TILE;
        offsets(t0, off);
        load_tile<GEO, R, NT>(bufA, Kb, Vb, off);
        while (t0 < row1) {
            offsets(t0 + STEP, off);
            load_tile<GEO, R, NT>(bufB, Kb, Vb, off);
            consume(bufA, t0, t0 - row0);
            t0 += STEP;
            if (t0 >= row1) break;
            offsets(t0 + STEP, off);
            load_tile<GEO, R, NT>(bufA, Kb, Vb, off);
            consume(bufB, t0, t0 - row0);
            t0 += STEP;
        }
    }

    HYLRA_TS(1);
    if (!DYN) {
        __syncthreads();                         // every score of the split is in LDS
        // row0 and the score stride are multiples of 4 floats: 16-byte stores are aligned
        float* __restrict__ dst = srow + row0;
        const int n = max(row1 - row0, 0);
        for (int i = 4 * tid; i < n; i += 4 * NW * 64) {
            if (i + 4 <= n) {
                *reinterpret_cast<float4*>(dst + i) = *reinterpret_cast<const float4*>(s_scores + i);
            } else {
                for (int e = i; e < n; ++e) dst[e] = s_scores[e];
            }
            if (bins)
                for (int e = i; e < min(i + 4, n); ++e) hist_add(s_hist, s_scores[e]);
        }
    }

    // the pair's partials: [head of the group][partial] from slot0 * G on
    const int n_part = DYN ? my_wgs * p.n_segs : p.n_splits;
    block_merge_store<GEO, NW>(st, smem, p.part_ml + (slot0 * G + split) * 2, (int64_t)n_part * 2,
                               p.part_acc + (slot0 * G + split) * D, (int64_t)n_part * D);
    __syncthreads();                             // between the last count and the flush
    if (bins) hist_flush<NW * 64>(s_hist, p.ghist + ((int64_t)b * p.Hkv + g) * kScoreBins);
    HYLRA_TS(2);
}

// Lane layout per (D, G): two 16-byte pieces per lane while the accumulators still fit a
// two-waves-per-SIMD register budget, one piece for the larger groups.
template <int D, int G>
struct FullCfg {
    static constexpr int CH = (D == 128 && G <= 4) ? 2 : 1;
};

// variant = 10 * MODE + R  (R = row groups per tile)
#define HYLRA_FULL_VARIANTS(X) X(2, 3) X(4, 3)
constexpr int kDefaultFullVariant = 23;

template <int D, int G>
static hipError_t launch_one(const FullParams& p, int B, int variant, hipStream_t st) {
    constexpr int CH = FullCfg<D, G>::CH;
    dim3 grid(p.n_splits, p.Hkv, B);
#define V(MODE, R)                                                                              \
    if (variant == 10 * MODE + R) {                                                             \
        hipLaunchKernelGGL((full_attn_split_kernel<D, G, CH, R, MODE>), grid, dim3(256),        \
                           p.rows_per_split * sizeof(float) + p.tbl_cap * sizeof(int), st, p);  \
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
