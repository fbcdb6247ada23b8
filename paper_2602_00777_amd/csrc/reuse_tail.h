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
    float M = NEG_BIG, num = 0.f, den = 0.f;
#pragma unroll
    for (int s = 0; s < SB; ++s) M = fmaxf(M, m_s[s]);
#pragma unroll
    for (int s = 0; s < SB; ++s) {
        const float w = s < S ? fast_exp2(m_s[s] - M) : 0.f;
        den = fmaf(w, l_s[s], den);
        num = fmaf(w, a_s[s], num);
    }
    return den > 0.f ? num / den : 0.f;
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
            float M = NEG_BIG, num = 0.f, den = 0.f;
#pragma unroll 8
            for (int s = 0; s < S; ++s) M = fmaxf(M, coherent_load(ml + 2 * s));
#pragma unroll 8
            for (int s = 0; s < S; ++s) {
                const float w = fast_exp2(coherent_load(ml + 2 * s) - M);
                den = fmaf(w, coherent_load(ml + 2 * s + 1), den);
                num = fmaf(w, coherent_load(acc + (int64_t)s * D), num);
            }
            p.out[(head0 + h) * D + col] = den > 0.f ? num / den : 0.f;
        }
    }
    HYLRA_TS(6);
    if (tid == 0) __hip_atomic_store(p.counters + pair, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace hylra
