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
    int gave_up;                    // a wave's bounded wait for a slot ran out (reported to the host, see FullParams::err_word)
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

// After the streaming loop (and a barrier): a workgroup in which a wave gave up waiting has
// left rows out, and its segment's counter may not return to zero -- nothing of the launch can
// be trusted.  The host is told through a word in pinned host memory that every later call on
// the context looks at (hylra_reset clears it and the counters).
DEVI void report_give_up(const ChunkQueue& cq, int* err_word) {
    if (threadIdx.x == 0 && cq.gave_up && err_word)
        __hip_atomic_store(err_word, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

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
        if (!have && !lds_load(&cq.done) && lane == 0)
            __hip_atomic_store(&cq.gave_up, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
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

// Segment and chunk arithmetic: host_logic.h (SegInfo, seg_chunks, chunk_bound, pair_segment,
// paired_unit), here bound to the launch's table.
DEVI void seg_chunks(const FullParams& p, SegInfo& sg) { seg_chunks(p.chunk_tile, p.n_chunks, sg); }
DEVI int chunk_bound(const FullParams& p, const SegInfo& sg, int c) { return chunk_bound(p.chunk_tile, sg, c); }

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
