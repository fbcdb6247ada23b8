// Wave-level core shared by the Full (streaming) and Reuse (gather) kernels.
//
// A wave64 works on "row groups": LPR = D / (8*CH) lanes share one KV row, each lane
// holding CH 16-byte pieces (8 bf16 each) of it, so one wave-wide load instruction reads
// RPG = 64 / LPR rows.  Every lane keeps an independent online-softmax state (running
// max m in log2 units, running sum l, unnormalised accumulator acc) per query head of the
// group for the subsequence of rows it has seen; states are merged once per workgroup.
//
// The score of a row is Eq. 1's q.K_j / sqrt(d); the weight update is the usual
// max-subtracted softmax of Eq. 1 evaluated incrementally (Algorithm 2, "standard full
// attention output" / "sparse attention output").
#pragma once
#include "device_util.h"

namespace hylra {

template <int D_, int G_, int CH_>
struct Geo {
    static constexpr int D = D_;               // head_dim
    static constexpr int G = G_;               // query heads per KV head
    static constexpr int CH = CH_;             // 16-byte pieces of a row per lane
    static constexpr int LPR = D / (8 * CH);   // lanes per row
    static constexpr int RPG = 64 / LPR;       // rows per wave-wide load
    static constexpr int ACC = 8 * CH;         // accumulator columns per lane per head
    static_assert(LPR == 4 || LPR == 8 || LPR == 16, "unsupported lane layout");
};

template <class GEO>
struct LaneState {
    float m[GEO::G];
    float l[GEO::G];
    float acc[GEO::G][GEO::ACC];
    DEVI void init() {
#pragma unroll
        for (int h = 0; h < GEO::G; ++h) {
            m[h] = NEG_BIG;
            l[h] = 0.f;
#pragma unroll
            for (int e = 0; e < GEO::ACC; ++e) acc[h][e] = 0.f;
        }
    }
};

// q of the group, as this lane's pieces: qv[h][j] = 8 bf16 at column (chunk + j*LPR)*8.
template <class GEO>
DEVI void load_q(uint4 (&qv)[GEO::G][GEO::CH], const uint16_t* __restrict__ q_group, int chunk) {
#pragma unroll
    for (int h = 0; h < GEO::G; ++h)
#pragma unroll
        for (int j = 0; j < GEO::CH; ++j)
            qv[h][j] = *reinterpret_cast<const uint4*>(q_group + h * GEO::D + (chunk + j * GEO::LPR) * 8);
}

// Register image of one tile: R row groups of K and of V, CH 16-byte pieces each.
template <class GEO, int R>
struct TileBuf {
    uint4 k[R][GEO::CH];
    uint4 v[R][GEO::CH];
};

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// 16-byte load; NT marks the line as streaming (K and V rows are read once and never again,
// so they should not displace anything in L2 / the memory-side cache).
template <bool NT>
DEVI uint4 load16(const uint16_t* __restrict__ p) {
    if (NT) {
        const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
        return make_uint4(t.x, t.y, t.z, t.w);
    }
    return *reinterpret_cast<const uint4*>(p);
}

// Issue the loads of one tile.  off[r] is the element offset (from K and from V) of this
// lane's first piece of its row in group r.
template <class GEO, int R, bool NT>
DEVI void load_tile(TileBuf<GEO, R>& b, const uint16_t* __restrict__ K,
                    const uint16_t* __restrict__ V, const int64_t (&off)[R]) {
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int j = 0; j < GEO::CH; ++j)
            b.k[r][j] = load16<NT>(K + off[r] + j * GEO::LPR * 8);
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int j = 0; j < GEO::CH; ++j)
            b.v[r][j] = load16<NT>(V + off[r] + j * GEO::LPR * 8);
}

// Consume one loaded tile.  valid[r] is consulted only when MASKED.  mean_s[r] receives the
// group-mean scaled score of that row (natural units).
template <class GEO, int R, bool MASKED>
DEVI void compute_tile(LaneState<GEO>& st, const uint4 (&qv)[GEO::G][GEO::CH],
                       const TileBuf<GEO, R>& b, const bool (&valid)[R], float scale_log2,
                       float scale_mean, float (&mean_s)[R]) {
    constexpr int G = GEO::G, CH = GEO::CH, LPR = GEO::LPR;
    const uint4 (&kr)[R][CH] = b.k;
    const uint4 (&vr)[R][CH] = b.v;

    float t[R][G];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        float sum_h = 0.f;
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float s = 0.f;
#pragma unroll
            for (int j = 0; j < CH; ++j) {
                s = dot2_bf16(kr[r][j].x, qv[h][j].x, s);
                s = dot2_bf16(kr[r][j].y, qv[h][j].y, s);
                s = dot2_bf16(kr[r][j].z, qv[h][j].z, s);
                s = dot2_bf16(kr[r][j].w, qv[h][j].w, s);
            }
            s = group_sum<LPR>(s);
            sum_h += s;
            t[r][h] = MASKED ? (valid[r] ? s * scale_log2 : NEG_BIG) : s * scale_log2;
        }
        mean_s[r] = sum_h * scale_mean;
    }

    // running maximum; rescale only when some lane of the wave saw a larger score
    float m_new[G];
    bool grow = false;
#pragma unroll
    for (int h = 0; h < G; ++h) {
        float mx = t[0][h];
#pragma unroll
        for (int r = 1; r < R; ++r) mx = fmaxf(mx, t[r][h]);
        m_new[h] = fmaxf(st.m[h], mx);
        grow |= m_new[h] > st.m[h];
    }
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {
#pragma unroll
        for (int h = 0; h < G; ++h) {
            const float alpha = fast_exp2(st.m[h] - m_new[h]);
            st.m[h] = m_new[h];
            st.l[h] *= alpha;
#pragma unroll
            for (int e = 0; e < GEO::ACC; ++e) st.acc[h][e] *= alpha;
        }
    }

    float p[R][G];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float w = fast_exp2(t[r][h] - st.m[h]);
            if (MASKED) w = valid[r] ? w : 0.f;
            p[r][h] = w;
            st.l[h] += w;
        }

#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const uint32_t w4[4] = {vr[r][j].x, vr[r][j].y, vr[r][j].z, vr[r][j].w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float v0 = bf16_lo(w4[i]), v1 = bf16_hi(w4[i]);
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    st.acc[h][j * 8 + 2 * i] = fmaf(p[r][h], v0, st.acc[h][j * 8 + 2 * i]);
                    st.acc[h][j * 8 + 2 * i + 1] = fmaf(p[r][h], v1, st.acc[h][j * 8 + 2 * i + 1]);
                }
            }
        }
}

// Load and consume one tile in one go.
template <class GEO, int R, bool MASKED, bool NT = false>
DEVI void attend_tile(LaneState<GEO>& st, const uint4 (&qv)[GEO::G][GEO::CH],
                      const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
                      const int64_t (&off)[R], const bool (&valid)[R], float scale_log2,
                      float scale_mean, float (&mean_s)[R]) {
    TileBuf<GEO, R> b;
    load_tile<GEO, R, NT>(b, K, V, off);
    compute_tile<GEO, R, MASKED>(st, qv, b, valid, scale_log2, scale_mean, mean_s);
}

// Floats of LDS that block_merge_store needs for a workgroup of NW waves.
template <class GEO, int NW>
constexpr int merge_smem_floats() {
    return NW * GEO::G * (GEO::D + 2);
}

// Merge the lane states of a whole workgroup (NW waves) into one partial per head and
// store it:  part_ml[h*ml_stride + {0,1}] = (max in log2 units, sum),
//            part_acc[h*acc_stride + 0..D-1] = unnormalised accumulator.
// Every thread of the workgroup must call this.  With COHERENT the partial is written with
// device-scope write-through stores, so that another workgroup can read it in the same
// launch (see coherent_load) without a full cache write-back.
//
// All workgroups of a launch reach this point at about the same time, so nothing overlaps
// it: it is kept short.  Within a wave the lanes that hold the same columns (one per row
// slot) are summed with register exchanges only: a halving butterfly over the four 16-lane
// rows (each step hands half of the values to the partner rows, so the work halves too),
// then rotations inside a row.  The waves meet once, in LDS, each with its own maximum.
template <class GEO, int NW, bool COHERENT = false>
DEVI void block_merge_store(LaneState<GEO>& st, float* smem, float* __restrict__ part_ml,
                            int64_t ml_stride, float* __restrict__ part_acc, int64_t acc_stride) {
    constexpr int G = GEO::G, D = GEO::D, LPR = GEO::LPR, ACC = GEO::ACC;
    constexpr int PER = ACC + 1;                       // summed values per head: accumulators, l
    constexpr int NV = (G * PER + 3) / 4 * 4;          // padded so that it halves twice
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunk = lane % LPR;
    float* s_max = smem;                    // [NW][G]
    float* s_l = smem + NW * G;             // [NW][G]
    float* s_acc = smem + 2 * NW * G;       // [NW][G][D]

    // the wave's maximum per head; every lane rescales its state to it
    float v[NV];
    float wmax[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        wmax[h] = strided_minmax<LPR, true>(st.m[h]);
        const float f = fast_exp2(st.m[h] - wmax[h]);
#pragma unroll
        for (int e = 0; e < ACC; ++e) v[h * PER + e] = st.acc[h][e] * f;
        v[h * PER + ACC] = st.l[h] * f;
    }
#pragma unroll
    for (int i = G * PER; i < NV; ++i) v[i] = 0.f;

    // rows 0,1 keep values [0, NV/2), rows 2,3 take [NV/2, NV); then even rows keep the lower
    // half of what they hold and odd rows the upper half
#pragma unroll
    for (int i = 0; i < NV / 2; ++i) {
        swap_rows32(v[i], v[i + NV / 2]);
        v[i] += v[i + NV / 2];
    }
#pragma unroll
    for (int i = 0; i < NV / 4; ++i) {
        swap_rows16(v[i], v[i + NV / 4]);
        v[i] += v[i + NV / 4];
        if (LPR <= 8) v[i] += dpp_move<0x128>(v[i]);       // row_ror:8
        if (LPR <= 4) v[i] += dpp_move<0x124>(v[i]);       // row_ror:4
    }
    // lane row r now holds values i + first, i < NV/4, summed over the whole wave
    const int row = lane >> 4;
    const int first = (row & 1) * (NV / 4) + (row >> 1) * (NV / 2);
    if ((lane & 15) < LPR) {
#pragma unroll
        for (int i = 0; i < NV / 4; ++i) {
            const int j = first + i;
            const int h = j / PER, e = j - h * PER;
            if (j < G * PER) {
                if (e < ACC) s_acc[(wave * G + h) * D + ((e >> 3) * LPR + chunk) * 8 + (e & 7)] = v[i];
                else if (chunk == 0) s_l[wave * G + h] = v[i];
            }
        }
    }
    if (lane == 0) {
#pragma unroll
        for (int h = 0; h < G; ++h) s_max[wave * G + h] = wmax[h];
    }
    __syncthreads();

    for (int i = tid; i < G * D; i += NW * 64) {
        const int h = i / D, col = i - h * D;
        float M = s_max[h];
#pragma unroll
        for (int w = 1; w < NW; ++w) M = fmaxf(M, s_max[w * G + h]);
        float a = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) a = fmaf(fast_exp2(s_max[w * G + h] - M), s_acc[(w * G + h) * D + col], a);
        if (COHERENT) coherent_store(part_acc + h * acc_stride + col, a);
        else part_acc[h * acc_stride + col] = a;
    }
    if (tid < G) {
        float M = s_max[tid];
#pragma unroll
        for (int w = 1; w < NW; ++w) M = fmaxf(M, s_max[w * G + tid]);
        float lsum = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) lsum = fmaf(fast_exp2(s_max[w * G + tid] - M), s_l[w * G + tid], lsum);
        if (COHERENT) {
            coherent_store(part_ml + tid * ml_stride, M);
            coherent_store(part_ml + tid * ml_stride + 1, lsum);
        } else {
            part_ml[tid * ml_stride] = M;
            part_ml[tid * ml_stride + 1] = lsum;
        }
    }
}

}  // namespace hylra
