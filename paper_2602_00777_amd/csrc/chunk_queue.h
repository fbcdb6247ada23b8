// Run-time distribution of the rows of a (batch, KV head) over its workgroups and their waves
// (guided self-scheduling), used by the streaming kernels of the Full layer.
//
// Compute units do not stream at the same speed (XCDs differ, and so do the units of one XCD),
// and with a fixed split the slowest workgroup sets the kernel time.  Here the wave tiles of a
// pair (a tile = the rows one wave loads at a time) are cut into segments, one per group of
// wgs_per_seg workgroups, and every segment into chunks of decreasing size (host-made table,
// the same for every pair).  The workgroups of a segment start on one chunk each and claim
// further ones from a device-scope counter, one claim per chunk: few enough that the counter
// is never contended.  Inside a workgroup the waves draw tiles of the current chunks from a
// ticket counter in LDS, so the waves of a workgroup also finish together.  The wave that
// draws the first tile of a chunk issues the claim for the workgroup's next chunk and looks at
// the result one tile later (memory returns loads and atomics in order, so by then it is
// there): nothing in the streaming loop waits for anything but the tile to be consumed.  The
// counter returns to zero by itself: every launch adds to it exactly n times per segment, n
// being the segment's chunks (n - S claims that succeed and one that fails per workgroup; with
// more than n workgroups, the first n fail once and the others neither start on a chunk nor
// claim), and the claim that draws the last value stores zero.
#pragma once
#include "device_util.h"
#include "launch.h"

namespace hylra {

struct ChunkQueue {
    int ticket;                     // next tile ticket of the workgroup
    int n_ready;                    // published slots
    int done;                       // no further slot will be published
    int first[kMaxChunks + 2];      // first[i] = first ticket of slot i; first[n_ready] = end
    int tile0[kMaxChunks + 1];      // first tile (of the pair's tiles) of slot i
};

// A drawn tile: its number among the pair's tiles (-1: none) and its ticket.
struct TileRef {
    int tile;                       // in a vector register, see next_tile
    int ticket;
};

// A claim on the pair's chunk counter that is under way: the atomic has been issued, its
// result has not been looked at yet.
struct PendingClaim {
    int raw;                        // lane 0: what the counter returned
    int slot;                       // the slot the new chunk becomes; -1: nothing pending
    int first;                      // its first ticket
};

// LDS words of the queue are read by every lane (one address: a broadcast) and moved to a
// scalar register, so the queue logic runs on the scalar unit and costs no vector registers.
// Ordering between the waves of the workgroup is by fences on LDS alone ("local"): a plain
// workgroup-scope acquire or release would also wait for the wave's loads from memory, i.e.
// for the tile it has just requested.
DEVI int lds_load(const int* p) {
    return __builtin_amdgcn_readfirstlane(__hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
}
DEVI int lds_load_acquire(const int* p) {
    const int v = lds_load(p);
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    return v;
}
DEVI void lds_store_release(int* p, int v) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// A wave's view of the queue: the slot it draws from, cached in scalar registers, so that a
// draw inside the slot costs one LDS operation (the ticket).
struct QueueCursor {
    int slot, first, next, tile0;   // tickets first .. next - 1 are tiles tile0 .. of slot `slot`
};

// Next tile of the pair for the calling wave (every lane gets the same answer), or -1 when
// the workgroup has none left.  Every wait here ends: a slot is published by a running wave
// of this workgroup that waits for nothing but its own memory operations, and the spin is
// bounded on top of that.  A wave that draws the first tile of a slot issues the claim for
// the workgroup's next chunk into pc (at most one claim per wave is under way: the caller
// publishes pc before it draws again).
DEVI TileRef next_tile(ChunkQueue& cq, int* __restrict__ ctr, QueueCursor& cur, PendingClaim& pc, int lane) {
    int T = 0;
    if (lane == 0) T = __hip_atomic_fetch_add(&cq.ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    T = __builtin_amdgcn_readfirstlane(T);
    int tile = -1;
    if (T >= cur.next) {
        // past the cached slot: wait until the ticket's slot is published, then walk to it
        bool have = false;
        for (int spin = 0; spin < (1 << 22); ++spin) {
            const int done = lds_load_acquire(&cq.done);
            const int nr = lds_load_acquire(&cq.n_ready);
            if (T < lds_load(&cq.first[nr])) {
                have = true;
                break;
            }
            if (done) break;
            __builtin_amdgcn_s_sleep(2);
        }
        if (have) {
            while (T >= cur.next) {
                ++cur.slot;
                cur.first = cur.next;
                cur.next = lds_load(&cq.first[cur.slot + 1]);
            }
            cur.tile0 = lds_load(&cq.tile0[cur.slot]);
        }
    }
    if (T < cur.next) {
        tile = cur.tile0 + (T - cur.first);
        if (T == cur.first) {
            if (lane == 0) pc.raw = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            pc.slot = cur.slot + 1;
            pc.first = cur.next;
        }
    }
    // Handed back in a vector register the compiler cannot prove uniform: with a provably
    // uniform row number it turns the consumer's "whole tile inside the cache?" test into
    // scalar control flow, duplicates the loop body around it and runs out of registers.
    TileRef r;
    asm volatile("v_mov_b32 %0, %1" : "=v"(r.tile) : "s"(tile));
    r.ticket = T;
    return r;
}

// The workgroup's segment for its sequence: first tile, number of tiles, and the number of
// tiles the host's chunk table was made for.  A full-length sequence has that many or one more
// (the last chunk then runs to the segment's end).  A shorter one uses the end of the table:
// guided self-scheduling cuts the next chunk from what remains, so the table's chunks from the
// one that holds tile `off` = made_for - tiles on are the table of a segment of `tiles` tiles
// (its first chunk clipped), with the same smallest chunk; the segment has n_eff chunks,
// table entries c0 .. n_chunks - 1.
struct SegInfo {
    int tile0, tiles, made_for;
    int wgs;                        // workgroups that serve the segment
    int off, c0, n_eff;             // set by seg_chunks()
};

// Every thread calls this (the result is the same for all and lives in scalar registers).
DEVI void seg_chunks(const FullParams& p, SegInfo& sg) {
    sg.off = max(sg.made_for - sg.tiles, 0);
    int lo = 0, hi = sg.off ? p.n_chunks : 0;       // largest c with chunk_tile[c] <= off (0 for a full-length sequence)
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (p.chunk_tile[mid] <= sg.off) lo = mid;
        else hi = mid - 1;
    }
    sg.c0 = lo;
    sg.n_eff = p.n_chunks - lo;
}

// Workgroup x of a grid of 2 * half workgroups -> the group of S workgroups (S even) it belongs
// to and its rank there: group u is made of the S / 2 workgroups u * S / 2 .. of the first half
// and of the S / 2 workgroups of the second half that sit one group further on (so that its
// workgroups of the second half land on other XCDs than those of the first half).
DEVI void paired_unit(int x, int half, int S, int& unit, int& w) {
    const int h = S >> 1;
    const int late = x >= half;
    int r = x - (late ? half : 0);
    if (late) r = r >= h ? r - h : r - h + half;
    unit = r / h;
    w = (late ? h : 0) + (r - unit * h);
}

// A pair that was dealt n workgroups of its own (sequences of different lengths): they form
// max(1, n / S) segments of S .. 2 S - 1 workgroups each (fewer than S only when n < S), S being
// the number of workgroups the chunk table was made for, so that a workgroup's first chunk
// (1 / (2 S) of its segment) stays below its fair share.  For workgroup w of the pair: its
// segment, its rank in it, the segment's workgroups and the rank of the segment's first one.
struct PairSeg {
    int seg, w, wgs, wg0;
};
DEVI PairSeg pair_segment(int n, int S, int w) {
    const int n_seg = max(1, n / S), base = n / n_seg, extra = n - base * n_seg;   // `extra` segments have one more
    PairSeg r;
    if (w < extra * (base + 1)) {
        r.seg = w / (base + 1), r.wgs = base + 1, r.wg0 = r.seg * (base + 1);
    } else {
        const int v = w - extra * (base + 1);
        r.seg = extra + v / base, r.wgs = base, r.wg0 = extra * (base + 1) + (r.seg - extra) * base;
    }
    r.w = w - r.wg0;
    return r;
}

// First tile (within the segment) of the segment's chunk c (0 .. n_eff - 1); chunk c is
// [chunk_bound(c), chunk_bound(c + 1)).
DEVI int chunk_bound(const FullParams& p, const SegInfo& sg, int c) {
    if (c >= sg.n_eff) return sg.tiles;
    return max(p.chunk_tile[sg.c0 + c] - sg.off, 0);
}

// One lane only.  raw: what the segment's counter returned to a claim of this workgroup.
// Returns the claimed chunk and its bounds, or -1 if the counter has run out.  Should a chunk
// be empty, the lane claims again (and waits for it) until a chunk has tiles or the counter
// runs out, so that every workgroup still ends with exactly one failed claim.  The counter returns to zero here: the
// claim that draws the last value of the launch stores zero.
DEVI int settle_claim(const FullParams& p, const SegInfo& sg, int* __restrict__ ctr, int raw, int& lo, int& hi) {
    for (;;) {
        if (raw == sg.n_eff - 1) __hip_atomic_store(ctr, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int c = sg.wgs + raw;
        if (c >= sg.n_eff) return -1;
        lo = chunk_bound(p, sg, c);
        hi = chunk_bound(p, sg, c + 1);
        if (hi > lo) return c;
        raw = __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Look at the result of the claim under way, if any, and publish it: the chunk as slot
// pc.slot of the queue, or the end of the queue.
DEVI void publish_claim(ChunkQueue& cq, const FullParams& p, int* __restrict__ ctr, PendingClaim& pc, int lane,
                        const SegInfo& sg) {
    if (pc.slot < 0) return;
    const int raw = __builtin_amdgcn_readfirstlane(pc.raw);
    if (lane == 0) {
        int lo = 0, hi = 0;
        if (settle_claim(p, sg, ctr, raw, lo, hi) >= 0) {
            cq.tile0[pc.slot] = sg.tile0 + lo;
            cq.first[pc.slot + 1] = pc.first + (hi - lo);
            lds_store_release(&cq.n_ready, pc.slot + 1);
        } else {
            lds_store_release(&cq.done, 1);
        }
    }
    pc.slot = -1;
}

}  // namespace hylra
