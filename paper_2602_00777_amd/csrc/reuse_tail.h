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
    for (int i = tid; i < G * D; i += NT) {
        const int h = i / D, col = i - h * D;
        const float* ml = p.part_ml + (head0 + h) * S * 2;
        const float* acc = p.part_acc + (head0 + h) * S * D + col;
        float M = NEG_BIG, num = 0.f, den = 0.f;
        if (S <= 16) {          // the usual case: every load of the merge is issued at once
            float m_s[16], l_s[16], a_s[16];
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                const bool on = s < S;
                m_s[s] = on ? coherent_load(ml + 2 * s) : NEG_BIG;
                l_s[s] = on ? coherent_load(ml + 2 * s + 1) : 0.f;
                a_s[s] = on ? coherent_load(acc + (int64_t)s * D) : 0.f;
            }
#pragma unroll
            for (int s = 0; s < 16; ++s) M = fmaxf(M, m_s[s]);
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                const float w = fast_exp2(m_s[s] - M);
                den = fmaf(w, l_s[s], den);
                num = fmaf(w, a_s[s], num);
            }
        } else {
#pragma unroll 8
            for (int s = 0; s < S; ++s) M = fmaxf(M, coherent_load(ml + 2 * s));
#pragma unroll 8
            for (int s = 0; s < S; ++s) {
                const float w = fast_exp2(coherent_load(ml + 2 * s) - M);
                den = fmaf(w, coherent_load(ml + 2 * s + 1), den);
                num = fmaf(w, coherent_load(acc + (int64_t)s * D), num);
            }
        }
        p.out[(head0 + h) * D + col] = den > 0.f ? num / den : 0.f;
    }
    HYLRA_TS(6);
    if (tid == 0) __hip_atomic_store(p.counters + pair, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace hylra
