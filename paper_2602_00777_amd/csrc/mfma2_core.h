// Second matrix-core form of a wave's work on a group of 32 KV rows (head_dim 128), shared by
// the Reuse kernel (reuse_mfma2.hip) and the Full kernel (full_mfma2.hip):
//
//   K rows   contracted with q by v_mfma_f32_16x16x32_bf16 with lane = row of a 16-row block,
//            which taken literally makes every load instruction touch 16 rows with only 64
//            bytes each.  Instead lanes n and n ^ 8 fetch the two halves of one 128-byte line
//            of the same row, and a row_ror:8 register move per loaded dword (own_row) then
//            gives every lane the pieces of its own row.  The scores of a block come back as
//            lane = head, registers = rows 4 gq .. 4 gq + 3 of the block.
//   V rows   loaded with 16 lanes per row (one instruction reads four whole 256-byte rows):
//            lane (n, gq) fetches, for the two blocks a, b of the group, columns 8 n .. 8 n + 7
//            of rows 4 gq + j of a (j < 4) and of b (j >= 4) -- the same eight rows, in the
//            same order, that its score registers cover.  An 8 x 8 transpose inside the lane
//            (32 byte permutes, no cross-lane traffic) turns these into, per column 8 n + e,
//            eight rows packed in one register quad: the B operand of
//            out[h][8 n + e] += P[h][rows] V[rows][8 n + e]  on v_mfma_f32_16x16x32_bf16.
//   weights  fp32, split into a high and a low bf16 half (two MFMAs per column set), so they
//            carry 16 mantissa bits.
//
// Per 32 rows this needs 8 + 16 MFMAs where the first form (mfma_core.h) needs 56 (it
// transposes V through the matrix cores, 16 rows at a time, and contracts with the 16-deep
// instruction).
#pragma once
#include "mfma_core.h"

namespace hylra {

// (lo half of x) | (lo half of y) << 16   and the same for the high halves
DEVI uint32_t pack_lo(uint32_t x, uint32_t y) { return __builtin_amdgcn_perm(y, x, 0x05040100u); }
DEVI uint32_t pack_hi(uint32_t x, uint32_t y) { return __builtin_amdgcn_perm(y, x, 0x07060302u); }

DEVI uint32_t dword_of(const uint4& v, int w) { return w == 0 ? v.x : w == 1 ? v.y : w == 2 ? v.z : v.w; }

// Within every 16-lane row: the lanes of the banks in MASK (bit b = lanes 4b .. 4b+3) receive
// src from the lane 8 places away, the others keep old (v_mov_b32 with row_ror:8).
template <int MASK>
DEVI int rotate_in(int old, int src) { return __builtin_amdgcn_update_dpp(old, src, 0x128, 0xF, MASK, false); }

// k[2L], k[2L+1]: the two loads of line L as issued (see the K loads of the kernel).  On
// return k[s] is the lane's own row n, columns 32 s + 8 gq .. + 7, for s = 0..3.
DEVI void own_row(uint4 (&k)[4]) {
#pragma unroll
    for (int L = 0; L < 2; ++L) {
        const uint4 a = k[2 * L], b = k[2 * L + 1];
        k[2 * L] = make_uint4(rotate_in<0xC>(a.x, b.x), rotate_in<0xC>(a.y, b.y), rotate_in<0xC>(a.z, b.z), rotate_in<0xC>(a.w, b.w));
        k[2 * L + 1] = make_uint4(rotate_in<0x3>(b.x, a.x), rotate_in<0x3>(b.y, a.y), rotate_in<0x3>(b.z, a.z), rotate_in<0x3>(b.w, a.w));
    }
}

// v[j] = eight consecutive bf16 columns of row j (j = 0..7).  t[e] = column e of the eight rows.
DEVI void transpose8x8(const uint4 (&v)[8], uint4 (&t)[8]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        uint32_t w[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const uint32_t x = dword_of(v[2 * r], e >> 1), y = dword_of(v[2 * r + 1], e >> 1);
            w[r] = (e & 1) ? pack_hi(x, y) : pack_lo(x, y);
        }
        t[e] = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// Online-softmax state of a wave: m, l belong to head n (identical in the 4 lanes of a head);
// register j of acc[e] in lane (n, gq) holds out[head 4 gq + j][column 8 n + e].
struct State2 {
    float m, l;
    float4_t acc[8];
    DEVI void init() {
        m = NEG_BIG;
        l = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = float4_t{0.f, 0.f, 0.f, 0.f};
    }
};

// One group of 32 rows (blocks a and b).  ka / kb: this lane's pieces of its row of K in each
// block; v: its eight V pieces (rows 4 gq + j of a, then of b); mask_a / mask_b: bit r set if
// row r of the block takes part.  Sa / Sb receive the raw (unscaled) scores of head n for rows
// 4 gq .. 4 gq + 3 of block a / b (zero for padding heads).
template <int G>
DEVI void group32(State2& st, const uint4 (&ka)[4], const uint4 (&kb)[4], const uint4 (&v)[8],
                  const uint4 (&qb)[4], uint32_t mask_a, uint32_t mask_b, float scale_log2, int n, int gq,
                  float4_t& Sa, float4_t& Sb) {
    Sa = float4_t{0.f, 0.f, 0.f, 0.f};
    Sb = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        Sa = mfma_k32(ka[i], qb[i], Sa);
        Sb = mfma_k32(kb[i], qb[i], Sb);
    }
    float t[8];
    bool ok[8];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        ok[j] = n < G && ((mask_a >> (4 * gq + j)) & 1u);
        ok[4 + j] = n < G && ((mask_b >> (4 * gq + j)) & 1u);
        t[j] = ok[j] ? Sa[j] * scale_log2 : NEG_BIG;
        t[4 + j] = ok[4 + j] ? Sb[j] * scale_log2 : NEG_BIG;
    }
    float mx = fmaxf(fmaxf(fmaxf(t[0], t[1]), fmaxf(t[2], t[3])), fmaxf(fmaxf(t[4], t[5]), fmaxf(t[6], t[7])));
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(st.m, mx);
    if (__builtin_amdgcn_ballot_w64(m_new > st.m) != 0) {
        const float alpha = fast_exp2(st.m - m_new);
        st.m = m_new;
        st.l *= alpha;
        // register j of this lane accumulates head 4 gq + j, whose factor is in lane 4 gq + j
        float a4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) a4[j] = __shfl(alpha, 4 * gq + j, 64);
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
            for (int j = 0; j < 4; ++j) st.acc[e][j] *= a4[j];
    }
    float w[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        w[j] = ok[j] ? fast_exp2(t[j] - st.m) : 0.f;
        st.l += w[j];
    }
    uint4 p_hi, p_lo;
    split_weights(w[0], w[1], p_hi.x, p_lo.x);
    split_weights(w[2], w[3], p_hi.y, p_lo.y);
    split_weights(w[4], w[5], p_hi.z, p_lo.z);
    split_weights(w[6], w[7], p_hi.w, p_lo.w);
    uint4 vt[8];
    transpose8x8(v, vt);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        st.acc[e] = mfma_k32(p_hi, vt[e], st.acc[e]);
        st.acc[e] = mfma_k32(p_lo, vt[e], st.acc[e]);
    }
}

// The wave states of a workgroup into LDS (s_m, s_l: [NW][16]; s_acc: [NW][G][128]); ends with
// the barrier after which every thread may read them.
template <int G, int NW>
DEVI void stage_states2(State2& st, float (*s_m)[16], float (*s_l)[16], float* s_acc, int n, int gq) {
    constexpr int D = 128;
    const int wave = threadIdx.x >> 6;
    float l = st.l;
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    if (gq == 0) {
        s_m[wave][n] = st.m;
        s_l[wave][n] = l;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int h = 4 * gq + j;
        if (h < G) {
            float4* dst = reinterpret_cast<float4*>(s_acc + (wave * G + h) * D + 8 * n);
            dst[0] = make_float4(st.acc[0][j], st.acc[1][j], st.acc[2][j], st.acc[3][j]);
            dst[1] = make_float4(st.acc[4][j], st.acc[5][j], st.acc[6][j], st.acc[7][j]);
        }
    }
    __syncthreads();
}
// Head h of the workgroup after stage_states2: its maximum, its sum, its accumulator column.
template <int NW>
DEVI float staged_max(const float (*s_m)[16], int h) {
    float M = s_m[0][h];
#pragma unroll
    for (int w = 1; w < NW; ++w) M = fmaxf(M, s_m[w][h]);
    return M;
}
template <int NW>
DEVI float staged_sum(const float (*s_m)[16], const float (*s_l)[16], int h, float M) {
    float ls = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) ls = fmaf(fast_exp2(s_m[w][h] - M), s_l[w][h], ls);
    return ls;
}
template <int G, int NW>
DEVI float staged_acc(const float (*s_m)[16], const float* s_acc, int h, int col, float M) {
    float a = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) a = fmaf(fast_exp2(s_m[w][h] - M), s_acc[(w * G + h) * 128 + col], a);
    return a;
}

// Merge the wave states of a workgroup into one partial per head, as mfma_block_merge_store
// does for the first form (only the accumulator layout differs).
template <int G, int NW, bool COHERENT>
DEVI void merge_store2(State2& st, float (*s_m)[16], float (*s_l)[16], float* s_acc,
                       float* __restrict__ part_ml, int64_t ml_stride, float* __restrict__ part_acc,
                       int64_t acc_stride, int n, int gq) {
    constexpr int D = 128;
    const int tid = threadIdx.x;
    stage_states2<G, NW>(st, s_m, s_l, s_acc, n, gq);
    for (int i = tid; i < G * D; i += NW * 64) {
        const int h = i / D, col = i - h * D;
        const float a = staged_acc<G, NW>(s_m, s_acc, h, col, staged_max<NW>(s_m, h));
        if (COHERENT) coherent_store(part_acc + h * acc_stride + col, a);
        else part_acc[h * acc_stride + col] = a;
    }
    if (tid < G) {
        const float M = staged_max<NW>(s_m, tid);
        const float ls = staged_sum<NW>(s_m, s_l, tid, M);
        if (COHERENT) {
            coherent_store(part_ml + tid * ml_stride, M);
            coherent_store(part_ml + tid * ml_stride + 1, ls);
        } else {
            part_ml[tid * ml_stride] = M;
            part_ml[tid * ml_stride + 1] = ls;
        }
    }
}

}  // namespace hylra
