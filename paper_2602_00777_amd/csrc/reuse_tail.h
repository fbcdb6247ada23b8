// The cross-workgroup half of the Reuse layer: once a workgroup has written its partial with
// device-scope write-through stores, it bumps the arrival counter of its (batch, KV head);
// whoever arrives last reads all partials back with device-scope loads and writes the output.
// No device-scope fence is used on purpose: on this multi-XCD part such a fence writes back
// the whole L2 of the XCD and costs far more than the entire kernel.
#pragma once
#include "device_util.h"
#include "launch.h"

namespace hylra {

// Cache row behind slot `pos` of a (batch, KV head)'s selection.  Token level: the entry
// itself.  Block level (paper, block-level sparsity): slot pos is row pos % block of the
// block named by entry pos / block; the quotient comes from a multiply-high with
// ceil(2^32 / block), which is at most one too large for pos < 2^31.  Anything that is not a
// row of the cache comes back negative or >= N and is skipped by the caller.
DEVI int reuse_row(const ReuseParams& p, const int32_t* __restrict__ ib, int pos) {
    if (p.block == 1) return ib[pos];
    int t = (int)__umulhi((uint32_t)pos, p.block_magic);
    if (t * p.block > pos) --t;
    const int c = ib[t];
    return (unsigned)c < (unsigned)p.n_blocks ? c * p.block + (pos - t * p.block) : -1;
}

// Merge of SB >= n_splits partials for output element i of the KV head's G*D outputs, with
// every load of the merge in flight at once (the loads are device-scope and each is a trip to
// memory: issued one after the other they would add up).  Slots s >= S are read from the
// last real partial and weighted zero.
template <int D, int SB>
DEVI float merge_partials(const ReuseParams& p, int64_t head0, int i, int S) {
    const int h = i / D, col = i - h * D;
    const float* ml = p.part_ml + (head0 + h) * S * 2;
    const float* acc = p.part_acc + (head0 + h) * S * D + col;
    float m_s[SB], l_s[SB], a_s[SB];
#pragma unroll
    for (int s = 0; s < SB; ++s) {
        const int sc = min(s, S - 1);
        m_s[s] = coherent_load(ml + 2 * sc);
        l_s[s] = coherent_load(ml + 2 * sc + 1);
        a_s[s] = coherent_load(acc + (int64_t)sc * D);
    }
    float M = NEG_BIG;
#pragma unroll
    for (int s = 0; s < SB; ++s) M = fmaxf(M, m_s[s]);
    MergeSum sum;
#pragma unroll
    for (int s = 0; s < SB; ++s)
        if (s < S) sum.add(s, fast_exp2(m_s[s] - M), l_s[s], a_s[s]);
    return sum.result();
}

// Element offset of cache row `row` of the workgroup's sequence from the kernel's K / V base
// (which already holds the KV head, and the batch for a contiguous cache).  tbl: the
// sequence's row of the page table, or nullptr for a contiguous cache.
DEVI int64_t reuse_row_offset(const ReuseParams& p, const int32_t* __restrict__ tbl, int row) {
    return tbl ? paged_row_offset(p.map, tbl, row, p.sn) : (int64_t)row * p.sn;
}

// Append-then-attend in one launch (Algorithm 2 takes the caches with the current token in
// them).  The token's key / value rows, one per (batch, KV head), are not in the cache when
// the launch starts: every lane whose entry names the token's position reads k_new / v_new
// instead of the cache, and the pair's first workgroup writes the two rows into the cache for
// the launches that follow -- nothing in this launch reads what it writes.  row: the token's
// position = the sequence's length before the call, clamped to 0 .. N - 1 (-1: no append).
struct NewRow {
    int row;
    const uint16_t* k;      // the pair's new key / value row
    const uint16_t* v;
};
// n_rows: in, the rows of the sequence by p.map; out, the rows the attention covers.
template <int D>
DEVI NewRow reuse_new_row(const ReuseParams& p, int b, int64_t pair, int& n_rows) {
    NewRow nr;
    nr.row = -1, nr.k = nullptr, nr.v = nullptr;
    if (p.k_new) {
        nr.row = min(p.map.seq_lens ? n_rows : p.N - 1, p.N - 1);
        nr.k = p.k_new + pair * D, nr.v = p.v_new + pair * D;
        n_rows = nr.row + 1;
    }
    return nr;
}
// Kb / Vb: the kernel's K / V base of this (batch, KV head); threads 0 .. D/4 - 1 of the pair's
// first workgroup copy 16 bytes each.
template <int D>
DEVI void reuse_store_new_row(const ReuseParams& p, const NewRow& nr, const int32_t* __restrict__ tbl,
                              const uint16_t* Kb, const uint16_t* Vb, int split, int tid) {
    if (nr.row < 0 || split != 0 || tid >= D / 4) return;
    const int piece = tid % (D / 8);
    const bool is_v = tid >= D / 8;
    const int64_t off = reuse_row_offset(p, tbl, nr.row) + 8 * piece;
    uint16_t* dst = const_cast<uint16_t*>(is_v ? Vb : Kb) + off;
    *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>((is_v ? nr.v : nr.k) + 8 * piece);
}

// Every thread of the workgroup (NT threads) calls this after its partial stores were issued.
template <int G, int D, int NT>
DEVI void reuse_merge_tail(const ReuseParams& p, int64_t pair, int64_t head0, int* s_last) {
    const int tid = threadIdx.x;
    HYLRA_TS(3);
    wait_vmem();
    __syncthreads();
    HYLRA_TS(4);
    if (tid == 0)
        *s_last = __hip_atomic_fetch_add(p.counters + pair, 1, __ATOMIC_RELAXED,
                                        __HIP_MEMORY_SCOPE_AGENT) == p.n_splits - 1;
    __syncthreads();
    HYLRA_TS(5);
    if (!*s_last) return;
    const int S = p.n_splits;
    constexpr int ITER = (G * D + NT - 1) / NT;      // output elements per thread
    if (S <= 16) {
        // the usual case.  All elements of a thread are merged in one go (clamped index,
        // guarded store) so that their loads overlap too.
        float r[ITER];
#pragma unroll
        for (int it = 0; it < ITER; ++it) {
            const int i = min(tid + it * NT, G * D - 1);
            r[it] = S <= 2 ? merge_partials<D, 2>(p, head0, i, S)
                  : S <= 4 ? merge_partials<D, 4>(p, head0, i, S)
                  : S <= 8 ? merge_partials<D, 8>(p, head0, i, S)
                           : merge_partials<D, 16>(p, head0, i, S);
        }
#pragma unroll
        for (int it = 0; it < ITER; ++it) {
            const int i = tid + it * NT;
            if (i < G * D) p.out[head0 * D + i] = r[it];
        }
    } else {
        for (int i = tid; i < G * D; i += NT) {
            const int h = i / D, col = i - h * D;
            const float* ml = p.part_ml + (head0 + h) * S * 2;
            const float* acc = p.part_acc + (head0 + h) * S * D + col;
            float M = NEG_BIG;
#pragma unroll 8
            for (int s = 0; s < S; ++s) M = fmaxf(M, coherent_load(ml + 2 * s));
            MergeSum sum;
#pragma unroll 8
            for (int s = 0; s < S; ++s)
                sum.add(s, fast_exp2(coherent_load(ml + 2 * s) - M), coherent_load(ml + 2 * s + 1),
                        coherent_load(acc + (int64_t)s * D));
            p.out[(head0 + h) * D + col] = sum.result();
        }
    }
    HYLRA_TS(6);
    if (tid == 0) __hip_atomic_store(p.counters + pair, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---- Merge by packets ------------------------------------------------------------------------
// A second way across workgroups, for launches whose workgroups are all resident at once (the
// host checks: no more workgroups than compute units).  Instead of "store the partial, count
// the arrival, the last one merges everything" -- three dependent trips to memory after the
// last row, and a merge by ONE compute unit -- every workgroup of a (batch, KV head) is also
// the consumer of one slice of the output columns: workgroup c merges columns c D/S .. of all
// heads.  A producer sends consumer c a packet [G][2] (max, sum) + [G][D/S] (its accumulator's
// columns of c); every float travels in a 64-bit unit {value, tag} written and read with one
// 64-bit agent-scope atomic access, so a unit that reads tag = 1 carries its value: nothing
// else has to be ordered, no counter, no wait for stores to be acknowledged.  The consumer
// polls the S packets addressed to it (contiguous), keeps what is tagged, and writes zero over
// every unit it has taken, which is the state the next launch expects (a launch ends before
// the next one starts, so these stores are complete by then; every unit has one writer and
// one reader per launch).  The poll is bounded; if it runs out (which takes a fault elsewhere)
// the host is told through err_word and the context has to be reset.  The merge itself runs
// in partial order 0 .. S - 1 with the arithmetic of combine_kernel, bit for bit.
constexpr uint32_t kPacketFull = 1u;
constexpr int kPacketSpins = 1 << 18;

// Producer.  pk_pair: the pair's packets (layout: host_logic.h, PacketShape); max_of(h),
// sum_of(h, M), acc_of(h, col, M): the workgroup's merged state.  Every thread calls.
template <int G, int D, int NT, class FM, class FS, class FA>
DEVI void send_packets(uint64_t* __restrict__ pk_pair, int S, int split, FM max_of, FS sum_of, FA acc_of) {
    const int tid = threadIdx.x;
    const PacketShape ps = packet_shape(G, D, S);
    auto put = [](uint64_t* p, float v) {
        __hip_atomic_store(p, ((uint64_t)kPacketFull << 32) | __float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
    for (int i = tid; i < G * D; i += NT) {
        const int h = i / D, col = i - h * D;
        put(pk_pair + packet_acc_unit(ps, G, split, h, col), acc_of(h, col, max_of(h)));
    }
    for (int i = tid; i < S * G; i += NT) {
        const int c = i / G, h = i - c * G;
        const float M = max_of(h);
        put(pk_pair + packet_ml_unit(ps, c, split, h, 0), M);
        put(pk_pair + packet_ml_unit(ps, c, split, h, 1), sum_of(h, M));
    }
}

// Consumer.  s_pk: kPacketUnitsPerThread * NT floats of LDS.  Every thread calls.
template <int G, int D, int NT>
DEVI void reuse_packet_tail(const ReuseParams& p, uint64_t* __restrict__ pk_pair, int64_t head0, int split,
                            float* s_pk) {
    constexpr int U = kPacketUnitsPerThread;
    const int tid = threadIdx.x;
    const PacketShape ps = packet_shape(G, D, p.n_splits);
    const int S = ps.S, W = ps.W, PK = ps.PK, total = S * PK;
    const int nu = (total + NT - 1) / NT;                   // units per thread (<= U: the host checks)
    uint64_t* __restrict__ mine = pk_pair + packet_ml_unit(ps, split, 0, 0, 0);      // S packets, contiguous
    HYLRA_TS(4);
    // Every round reads all of the thread's units again, without branches, so that the loads of
    // a round are in flight together (a unit that was full stays full until this thread clears
    // it below; a place past the end loads the last unit and ignores it -- that unit's owner
    // may have cleared it already).
    uint64_t v[U];
    bool ok = false;
    for (int spin = 0; spin < kPacketSpins && !ok; ++spin) {
        if (spin) __builtin_amdgcn_s_sleep(1);
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (u < nu) v[u] = __hip_atomic_load(mine + min(tid + u * NT, total - 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ok = true;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (u < nu) ok = ok && (tid + u * NT >= total || (uint32_t)(v[u] >> 32) == kPacketFull);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (u < nu && tid + u * NT < total) {
            s_pk[tid + u * NT] = __uint_as_float((uint32_t)v[u]);
            __hip_atomic_store(mine + tid + u * NT, (uint64_t)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    if (!ok && p.err_word) __hip_atomic_store(p.err_word, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    __syncthreads();
    HYLRA_TS(5);
    // The merge, in the common order (MergeSum): S / 4 lanes per output element, one block of
    // four partials each; their maxima meet by exchange, their block sums are added in block
    // order by the element's first lane.  G W elements of S / 4 lanes = G D / 4 <= NT threads.
    static_assert(G * D / kMergeBlock <= NT, "one pass of the workgroup covers every element");
    const int L = S / kMergeBlock, ll = 31 - __clz(L), lw = 31 - __clz(W);      // (powers of two; S >= 4)
    const int e = tid >> ll, blk = tid & (L - 1);
    if (e < G * W) {                                    // (whole groups of L <= 32 lanes, inside one wave)
        const int h = e >> lw, j = e & (W - 1);
        const float* pk = s_pk + blk * kMergeBlock * PK;
        float m4[kMergeBlock], l4[kMergeBlock], a4[kMergeBlock];
#pragma unroll
        for (int i = 0; i < kMergeBlock; ++i) {
            m4[i] = pk[i * PK + 2 * h];
            l4[i] = pk[i * PK + 2 * h + 1];
            a4[i] = pk[i * PK + 2 * G + h * W + j];
        }
        float M = fmaxf(fmaxf(m4[0], m4[1]), fmaxf(m4[2], m4[3]));
        for (int x = 1; x < L; x <<= 1) M = fmaxf(M, __shfl_xor(M, x, 64));
        float db = 0.f, nb = 0.f;
#pragma unroll
        for (int i = 0; i < kMergeBlock; ++i) {
            const float w = fast_exp2(m4[i] - M);
            db = fmaf(w, l4[i], db);
            nb = fmaf(w, a4[i], nb);
        }
        float den = 0.f, num = 0.f;
        const int first = threadIdx.x & 63 & ~(L - 1);
        for (int x = 0; x < L; ++x) {
            den += __shfl(db, first + x, 64);
            num += __shfl(nb, first + x, 64);
        }
        if (blk == 0) p.out[(head0 + h) * D + split * W + j] = den > 0.f ? num / den : 0.f;
    }
    HYLRA_TS(6);
}

}  // namespace hylra
