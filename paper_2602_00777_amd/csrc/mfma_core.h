// Matrix-core building blocks shared by the Reuse and Full kernels: how one wave consumes a
// block of 16 KV rows with v_mfma_f32_16x16x32_bf16 / v_mfma_f32_16x16x16_bf16.
//
// Lane roles (wave64): n = lane & 15, gq = lane >> 4.
//   as loader      lane (n, gq) holds, for row n of the block, columns 32 i + 8 gq .. + 7
//   after scores   lane (n, gq) holds the scores of head n for rows 4 gq .. 4 gq + 3
//   accumulators   lane (n, gq) register j of tile t holds out[head 4 gq + j][column 16 t + n]
#pragma once
#include "device_util.h"

namespace hylra {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4m_t __attribute__((ext_vector_type(4)));

DEVI float4_t mfma_k32(uint4 a, uint4 b, float4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}
DEVI float4_t mfma_k16(uint2 a, uint2 b, float4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(short4_t, a),
                                                     __builtin_bit_cast(short4_t, b), c, 0, 0, 0);
}
// two fp32 values whose low 16 bits are dropped, packed as (lo half = a, hi half = b)
DEVI uint32_t pack_hi16(float a, float b) {
    return (__float_as_uint(a) >> 16) | (__float_as_uint(b) & 0xffff0000u);
}
// two fp32 values rounded to nearest-even bf16 (v_cvt_pk_bf16_f32), packed the same way
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
DEVI uint32_t pack_bf16_rne(float a, float b) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2_t){a, b}, bf16x2_t));
}
// Softmax weights as two bf16 operands of the P V contraction: w = hi + lo with hi = w rounded
// to bf16 and lo = the (signed) remainder rounded to bf16, i.e. 16 to 17 mantissa bits with a
// rounding error of at most 2^-18 w that has no preferred sign.  (Dropping low bits instead
// biases every weight downwards; the bias does not average out over the rows and showed as
// 5e-4 of the largest output component against 1e-5 for the fp32 vector kernels.)
DEVI void split_weights(float w0, float w1, uint32_t& p_hi, uint32_t& p_lo) {
    p_hi = pack_bf16_rne(w0, w1);
    p_lo = pack_bf16_rne(w0 - __uint_as_float(p_hi << 16), w1 - __uint_as_float(p_hi & 0xffff0000u));
}
template <bool NT>
DEVI uint4 ld16(const uint16_t* __restrict__ p) {
    if (NT) {
        const u32x4m_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4m_t*>(p));
        return make_uint4(t.x, t.y, t.z, t.w);
    }
    return *reinterpret_cast<const uint4*>(p);
}


// q as the B operand of the score MFMA: lane (head n, piece gq) holds q[n][32 i + 8 gq ..],
// zero for the padding heads n >= G.
template <int D, int G>
DEVI void mfma_load_q(uint4 (&qb)[D / 32], const uint16_t* __restrict__ q_group, int n, int gq) {
#pragma unroll
    for (int i = 0; i < D / 32; ++i)
        qb[i] = n < G ? *reinterpret_cast<const uint4*>(q_group + n * D + 32 * i + 8 * gq)
                      : make_uint4(0, 0, 0, 0);
}

// 0/1 selector operands: pushed through an MFMA with a 16x32 V tile as A, selector `half`
// returns columns 16*half .. 16*half+15 of the tile as lane = column, registers = 4 rows.
DEVI void mfma_selectors(uint4 (&sel)[2], int n, int gq) {
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        uint32_t w[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            const bool lo_on = (gq >> 1) == half && 8 * (gq & 1) + 2 * e2 == n;
            const bool hi_on = (gq >> 1) == half && 8 * (gq & 1) + 2 * e2 + 1 == n;
            w[e2] = (lo_on ? 0x3F80u : 0u) | (hi_on ? 0x3F800000u : 0u);      // bf16 1.0
        }
        sel[half] = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// Online-softmax state of one wave: m, l belong to head n (identical in the 4 lanes of a head);
// acc as described above.
template <int D>
struct MfmaState {
    float m, l;
    float4_t acc[D / 16];
    DEVI void init() {
        m = NEG_BIG;
        l = 0.f;
#pragma unroll
        for (int t = 0; t < D / 16; ++t) acc[t] = float4_t{0.f, 0.f, 0.f, 0.f};
    }
};

// One block of 16 rows.  kb / vb: this lane's pieces of its row of K and V.  vmask: bit r set
// if row r of the block takes part.  Returns the raw scores (unscaled dot products) of head n
// for rows 4 gq .. 4 gq + 3 (zero for padding heads).
template <int D, int G>
DEVI float4_t mfma_block(MfmaState<D>& st, const uint4 (&kb)[D / 32], const uint4 (&vb)[D / 32],
                         const uint4 (&qb)[D / 32], const uint4 (&sel)[2], uint32_t vmask,
                         float scale_log2, int n, int gq) {
    constexpr int KI = D / 32, TILES = D / 16;
    float4_t S = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < KI; ++i) S = mfma_k32(kb[i], qb[i], S);
    float t[4];
    bool ok[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        ok[j] = n < G && ((vmask >> (4 * gq + j)) & 1u);
        t[j] = ok[j] ? S[j] * scale_log2 : NEG_BIG;
    }
    float mx = fmaxf(fmaxf(t[0], t[1]), fmaxf(t[2], t[3]));
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
        for (int tl = 0; tl < TILES; ++tl)
#pragma unroll
            for (int j = 0; j < 4; ++j) st.acc[tl][j] *= a4[j];
    }
    float w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        w[j] = ok[j] ? fast_exp2(t[j] - st.m) : 0.f;
        st.l += w[j];
    }
    uint2 p_hi, p_lo;
    split_weights(w[0], w[1], p_hi.x, p_lo.x);
    split_weights(w[2], w[3], p_hi.y, p_lo.y);
#pragma unroll
    for (int i = 0; i < KI; ++i)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const float4_t T = mfma_k32(vb[i], sel[half], float4_t{0.f, 0.f, 0.f, 0.f});
            const uint2 vt = make_uint2(pack_hi16(T[0], T[1]), pack_hi16(T[2], T[3]));
            st.acc[2 * i + half] = mfma_k16(p_hi, vt, st.acc[2 * i + half]);
            st.acc[2 * i + half] = mfma_k16(p_lo, vt, st.acc[2 * i + half]);
        }
    return S;
}

// Merge the wave states of a workgroup of NW waves into one partial per head:
// (max, sum) to part_ml[h * ml_stride + {0,1}], accumulator to part_acc[h * acc_stride + col].
// s_m, s_l: [NW][16]; s_acc: [NW][G][D].  Every thread must call it.
template <int D, int G, int NW>
DEVI void mfma_stage_states(MfmaState<D>& st, float (*s_m)[16], float (*s_l)[16], float* s_acc, int n, int gq);

// A (batch, KV head) that ONE workgroup covers: its output straight from the staged wave states
// (s_m, s_l: [NW][16]; s_acc: [NW][G][D]; after the staging barrier), out: [G][D].  The same
// bits as the partial followed by a merge of one partial: there the weight is 2^0 = 1, and
// fma(1, x, 0) and 0 + x are x.
template <int D, int G, int NW>
DEVI void staged_to_output(const float (*s_m)[16], const float (*s_l)[16], const float* s_acc, float* __restrict__ out) {
    for (int i = threadIdx.x; i < G * D; i += NW * 64) {
        const int h = i / D, col = i - h * D;
        float M = s_m[0][h];
#pragma unroll
        for (int w = 1; w < NW; ++w) M = fmaxf(M, s_m[w][h]);
        float a = 0.f, ls = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float f = fast_exp2(s_m[w][h] - M);
            a = fmaf(f, s_acc[(w * G + h) * D + col], a);
            ls = fmaf(f, s_l[w][h], ls);
        }
        out[i] = ls > 0.f ? a / ls : 0.f;
    }
}

template <int D, int G, int NW, bool COHERENT>
DEVI void mfma_block_merge_store(MfmaState<D>& st, float (*s_m)[16], float (*s_l)[16],
                                 float* s_acc, float* __restrict__ part_ml, int64_t ml_stride,
                                 float* __restrict__ part_acc, int64_t acc_stride, int n, int gq) {
    const int tid = threadIdx.x;
    mfma_stage_states<D, G, NW>(st, s_m, s_l, s_acc, n, gq);
    for (int i = tid; i < G * D; i += NW * 64) {
        const int h = i / D, col = i - h * D;
        float M = s_m[0][h];
#pragma unroll
        for (int w = 1; w < NW; ++w) M = fmaxf(M, s_m[w][h]);
        float a = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) a = fmaf(fast_exp2(s_m[w][h] - M), s_acc[(w * G + h) * D + col], a);
        if (COHERENT) coherent_store(part_acc + h * acc_stride + col, a);
        else part_acc[h * acc_stride + col] = a;
    }
    if (tid < G) {
        float M = s_m[0][tid];
#pragma unroll
        for (int w = 1; w < NW; ++w) M = fmaxf(M, s_m[w][tid]);
        float ls = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) ls = fmaf(fast_exp2(s_m[w][tid] - M), s_l[w][tid], ls);
        if (COHERENT) {
            coherent_store(part_ml + tid * ml_stride, M);
            coherent_store(part_ml + tid * ml_stride + 1, ls);
        } else {
            part_ml[tid * ml_stride] = M;
            part_ml[tid * ml_stride + 1] = ls;
        }
    }
}

// The wave states of a workgroup into LDS; ends with the barrier after which every thread may
// read them.
template <int D, int G, int NW>
DEVI void mfma_stage_states(MfmaState<D>& st, float (*s_m)[16], float (*s_l)[16], float* s_acc, int n, int gq) {
    const int wave = threadIdx.x >> 6;
    float l = st.l;
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    if (gq == 0) {
        s_m[wave][n] = st.m;
        s_l[wave][n] = l;
    }
#pragma unroll
    for (int tl = 0; tl < D / 16; ++tl)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int h = 4 * gq + j;
            if (h < G) s_acc[(wave * G + h) * D + 16 * tl + n] = st.acc[tl][j];
        }
    __syncthreads();
}

}  // namespace hylra
