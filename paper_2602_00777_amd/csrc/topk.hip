// Full layer, after the streaming pass: merge of the split partials into the attention
// output (Algorithm 2, "O <- Softmax(S) V") and the EXACT selection of the k positions with
// the largest group-mean score (Algorithm 2, "I <- TopK(S, B)"; ties to the lower position,
// ascending order).
//
// Rows are ranked by (key descending, position ascending), key = the order-preserving 32-bit
// image of the fp32 score.  The selection is a radix select on the key, 12 + 12 + 8 bits, over
// chunks of 8192 rows, one workgroup of 1024 threads per chunk holding its rows in registers:
//   level 1  a histogram of the top 12 key bits over all of the pair's rows.  It is COMPLETE
//            when the first kernel here starts: the streaming kernel bins the scores it has
//            staged in LDS and adds its non-empty bins to the pair's histogram in memory (for the
//            kernels that do not, score_hist_kernel below does it in a launch of its own).
//   topk_scan_kernel   every chunk finds the level-1 threshold bin T1 (the bin that holds the
//            k-th best row), counts its rows in the bins above T1 (selected for sure) and lists
//            its rows of bin T1 (key, position; about 1.5 % of the rows) in memory.  One more
//            workgroup per (batch, KV head) merges the attention partials meanwhile.
//   topk_emit_kernel   every chunk reads the lists of all the pair's chunks (a few KB), bins them
//            on the next 12 key bits (level 2: bin T2), ranks the handful of rows whose top 24
//            bits equal (T1, T2) pairwise (level 3; with massive ties: one more histogram over
//            the last 8 bits, rows equal to the threshold key taken in position order), and
//            emits the selected rows of its chunk at the place the chunks before it leave.
// A workgroup reads its own chunk and those lists, nothing else: what bounds these kernels is
// what ONE compute unit can pull from beyond its L2 (about 20 GB/s: a workgroup that scans all
// 32768 rows of a pair spends 6 us on that alone, all 131072 rows 25 us -- measured with a
// one-launch form of this selection, which lost for that reason), so the work is cut so that no
// workgroup reads more than 32 KB of scores.  If a chunk has more rows in bin T1 than its list
// holds (heavy ties), the second kernel falls back to scanning all rows of the pair itself.
#include "launch.h"
#include "select_util.h"

namespace hylra {

constexpr int kTopkFineBins = 4096;
constexpr int kTopkList = 3072;       // rows of bin T1 (all chunks of a pair) a workgroup can hold in LDS
constexpr int E_OWN = kTopkChunkRows / (4 * SEL_THREADS);      // float4 groups per thread = 2
static_assert(E_OWN * 4 * SEL_THREADS == kTopkChunkRows, "a chunk is E_OWN float4 groups per thread");

// Threshold bin of a histogram whose bins NB-1-4t .. NB-4-4t sit in h4[0..3] of thread t: the
// bin T that holds the k-th largest row and the number of rows in the bins above it.  s_pick
// must hold (SEL_BINS, 0) on entry (what comes back when k = 0).  Two barriers; once per kernel
// (s_wave and s_pick are not reusable afterwards without another barrier).
DEVI void threshold_pick(const int (&h4)[4], int k, int* s_wave, int* s_pick, int& T, int& above) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int local = h4[0] + h4[1] + h4[2] + h4[3];
    const int incl = wave_incl_scan_dpp(local);
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    int excl = incl - local;
#pragma unroll
    for (int w = 0; w < SEL_WAVES; ++w) {
        const int t = s_wave[w];                 // (one address for all lanes: a broadcast)
        excl += w < wave ? t : 0;
    }
    if (excl < k && k <= excl + local) {
        int c = excl;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (c < k && k <= c + h4[e]) {
                s_pick[0] = SEL_BINS - 1 - (4 * tid + e);
                s_pick[1] = c;
            }
            c += h4[e];
        }
    }
    __syncthreads();
    T = s_pick[0];
    above = s_pick[1];
}

DEVI float f4_at(const float4& v, int e) { return e == 0 ? v.x : e == 1 ? v.y : e == 2 ? v.z : v.w; }

// Workgroups are handed to the XCDs (each with an L2 of its own) in turn, by their number:
// workgroup x runs on XCD x % 8.  The workgroups of a (batch, KV head) are numbered 8 apart, so
// that they share one L2 (the lists one kernel writes and the other reads, the pair's
// histogram).  Nothing but speed depends on where a workgroup really lands.  per_pair
// workgroups per pair; returns false for the padding workgroups of the last eight pairs.
DEVI bool xcd_pair_role(int per_pair, int64_t pairs, int64_t& pair, int& role) {
    const int slot = blockIdx.x >> 3;
    pair = (int64_t)(slot / per_pair) * 8 + (blockIdx.x & 7);
    role = slot % per_pair;
    return pair < pairs;
}

// The chunk's rows: register j of thread t holds float4 group first4 + j * 1024 + t.
struct ChunkRows {
    float4 v[E_OWN];
    int first4;
    DEVI void load(const float* sc, int n4, int c) {
        first4 = c * E_OWN * SEL_THREADS;
#pragma unroll
        for (int j = 0; j < E_OWN; ++j) {
            const int i = grp(j);
            v[j] = i < n4 ? reinterpret_cast<const float4*>(sc)[i] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    DEVI int grp(int j) const { return first4 + j * SEL_THREADS + (int)threadIdx.x; }
    DEVI uint32_t key(int j, int e) const { return ordered_key(f4_at(v[j], e)); }
};

// ---- scan: level-1 threshold, the chunk's count and list ----
// ONE: the one-launch form (topk_one_kernel): the list leaves with agent-scope stores, and once
// they are acknowledged a header {rows above T1, rows in T1} goes to every chunk of the pair.
constexpr int kTopkHdrBits = 14;        // both header fields are <= 8192
constexpr uint32_t kTopkHdrFull = 1u;
constexpr int kTopkHdrSpins = 1 << 18;
constexpr int kTopkOneMaxChunks = 256;  // chunks per pair the one-launch form is built for

template <bool ONE>
DEVI void scan_part(const TopkParams& p, int64_t pair, int c, const ChunkRows& rows, int N, int k, int& T1, int& above1) {
    __shared__ int s_wave[SEL_WAVES + 1];
    __shared__ int s_pick[2];
    __shared__ int s_n, s_above;
    __shared__ int2 s_list[kTopkChunkList];
    const int tid = threadIdx.x, lane = tid & 63;
    int h4[4];
    {
        const int4 h = *reinterpret_cast<const int4*>(p.ghist + pair * SEL_BINS + SEL_BINS - 4 - 4 * tid);
        h4[0] = h.w, h4[1] = h.z, h4[2] = h.y, h4[3] = h.x;
    }
    if (tid == 0) s_n = 0, s_above = 0, s_pick[0] = SEL_BINS, s_pick[1] = 0;
    HYLRA_TS_SEL(4);

    // ---- level 1: threshold bin of the complete histogram (the same in every chunk) ----
    threshold_pick(h4, k, s_wave, s_pick, T1, above1);
    HYLRA_TS_SEL(5);
    if (!ONE && c == 0 && tid == 0) p.pair_info[pair] = make_int2(T1, above1);

    // ---- the chunk's rows: above bin T1 (counted), in it (listed) ----
    const uint32_t lo_key = (uint32_t)T1 << 20, top_key = lo_key | 0xFFFFFu;      // bin T1 = [lo_key, top_key]
    int above = 0, mine = 0;
    uint32_t in_bin = 0;
#pragma unroll
    for (int j = 0; j < E_OWN; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (4 * rows.grp(j) + e >= N || T1 >= SEL_BINS) continue;
            const uint32_t key = rows.key(j, e);
            above += key > top_key;
            if (key >= lo_key && key <= top_key) in_bin |= 1u << (4 * j + e), ++mine;
        }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) above += __shfl_xor(above, m, 64);
    if (lane == 0 && above) atomicAdd(&s_above, above);
    HYLRA_TS_SEL(2);
    // list entries are reserved per wave: a prefix sum over the lanes and ONE atomic on the list's
    // counter (an atomic per lane on that single LDS address is served lane by lane: 1024 of them
    // took 2.6 us here)
    const int incl = wave_incl_scan_dpp(mine);
    int wave_base = 0;
    if (lane == 63) wave_base = atomicAdd(&s_n, incl);
    int slot = __shfl(wave_base, 63, 64) + incl - mine;
#pragma unroll
    for (int j = 0; j < E_OWN; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if ((in_bin >> (4 * j + e)) & 1u) {
                if (slot < kTopkChunkList) s_list[slot] = make_int2((int)rows.key(j, e), 4 * rows.grp(j) + e);
                ++slot;
            }
    HYLRA_TS_SEL(3);
    __syncthreads();
    HYLRA_TS_SEL(6);
    const int n = s_n;                           // may exceed the list: the emission then scans all rows
    const int64_t cslot = pair * p.max_chunks + c;
    int2* __restrict__ gl = p.chunk_list + cslot * kTopkChunkList;
    if (!ONE) {
        for (int i = tid; i < min(n, kTopkChunkList); i += SEL_THREADS) gl[i] = s_list[i];
        if (tid == 0) p.chunk_info[cslot] = make_int2(s_above, n);
    } else {
        // (entries as 64-bit agent-scope stores: the readers are other workgroups of this launch)
        for (int i = tid; i < min(n, kTopkChunkList); i += SEL_THREADS) {
            const int2 e = s_list[i];
            __hip_atomic_store(reinterpret_cast<uint64_t*>(gl + i), ((uint64_t)(uint32_t)e.y << 32) | (uint32_t)e.x,
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        wait_vmem();
        __syncthreads();                         // every entry of the list has been acknowledged
        const uint64_t hdr = ((uint64_t)kTopkHdrFull << 32) | ((uint32_t)s_above << kTopkHdrBits) | (uint32_t)n;
        const int MC = p.max_chunks;
        for (int t = tid; t < p.chunks; t += SEL_THREADS)
            __hip_atomic_store(p.headers + ((pair * MC + t) * MC + c), hdr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    HYLRA_TS_SEL(7);
}

// ---- merge of the attention partials (the pair's workgroups C .. C + merge_wgs - 1, or its
// chunk 0 in passing when merge_wgs = 0).  Returns true for a workgroup that has nothing else
// to do. ----
DEVI bool merge_part(const TopkParams& p, int64_t pair, int b, int g, int c) {
    const int C = p.chunks;
    const int tid = threadIdx.x;
    // ---- attention output (the pair's last merge_wgs workgroups): L lanes per output element,
    // each lane merging every L-th partial with the loads of four partials in flight at once,
    // then a log-sum-exp merge across the L lanes.  L and the number of workgroups are chosen
    // on the host so that a lane has at most four partials and a workgroup one sweep (every
    // further trip is another round to memory, and this is the kernel's longest chain). ----
    // (merge_wgs = 0: few partials, no workgroups to spare -- chunk 0 merges before it scans)
    if (c >= C || (p.merge_wgs == 0 && c == 0)) {
        const int merge_wgs = max(p.merge_wgs, 1), merge_id = c >= C ? c - C : 0;
        const PartView pv = part_view(p.pair_map, pair, p.n_splits);
        const int S = pv.S, D = p.D, G = p.G;
        const int64_t hb = pv.first * G;              // first partial of the pair's first head
        const int L = p.merge_lanes;
        const int64_t head0 = (int64_t)b * p.Hq + (int64_t)g * G;
        const int sub = tid & (L - 1), per_sweep = SEL_THREADS / L;
        const int share = (G * D + merge_wgs - 1) / merge_wgs;
        const int begin = merge_id * share, end = min(G * D, begin + share);
        for (int i0 = begin; i0 < end; i0 += per_sweep) {
            const int i = i0 + tid / L;
            const bool live = i < end;
            const int h = live ? i / D : 0, col = live ? i - h * D : 0;
            const float* ml = p.part_ml + (hb + (int64_t)h * S) * 2;
            const float* acc = p.part_acc + (hb + (int64_t)h * S) * D + col;
            float M = NEG_BIG, num = 0.f, den = 0.f;
            for (int s0 = sub; s0 < S; s0 += 4 * L) {
                float m_s[4], l_s[4], a_s[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int sx = min(s0 + u * L, S - 1);
                    const float2 t = *reinterpret_cast<const float2*>(ml + 2 * sx);
                    m_s[u] = s0 + u * L < S ? t.x : NEG_BIG;
                    l_s[u] = t.y;
                    a_s[u] = acc[(int64_t)sx * D];
                }
                const float M2 = fmaxf(fmaxf(fmaxf(m_s[0], m_s[1]), fmaxf(m_s[2], m_s[3])), M);
                const float r = fast_exp2(M - M2);
                num *= r, den *= r;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float w = s0 + u * L < S ? fast_exp2(m_s[u] - M2) : 0.f;
                    den = fmaf(w, l_s[u], den);
                    num = fmaf(w, a_s[u], num);
                }
                M = M2;
            }
            float Mg = M;
            for (int m = 1; m < L; m <<= 1) Mg = fmaxf(Mg, __shfl_xor(Mg, m, 64));
            const float r = fast_exp2(M - Mg);
            num *= r, den *= r;
            for (int m = 1; m < L; m <<= 1) {
                num += __shfl_xor(num, m, 64);
                den += __shfl_xor(den, m, 64);
            }
            if (live && sub == 0) p.out[(head0 + h) * D + col] = den > 0.f ? num / den : 0.f;
        }
    }
    return c >= C;

}

// ---- first kernel: level-1 threshold, counts and lists per chunk; merge of the partials ----
__global__ __launch_bounds__(SEL_THREADS) void topk_scan_kernel(TopkParams p) {
    const int C = p.chunks;
    int64_t pair;
    int c;
    if (!xcd_pair_role(C + p.merge_wgs, p.pairs, pair, c)) return;
    const int b = (int)(pair / p.Hkv), g = (int)(pair - (int64_t)b * p.Hkv);
    if (merge_part(p, pair, b, g, c)) return;

    // this sequence ranks its first N rows and selects k of them
    const int N = seq_units(p.seq_lens, b, p.N, p.sel_block), k = min(p.k, N);
    ChunkRows rows;
    rows.load(p.scores + pair * p.score_stride, (N + 3) >> 2, c);
    int T1, above1;
    scan_part<false>(p, pair, c, rows, N, k, T1, above1);
}

// ---- emission: levels 2 and 3, ordered output of the chunk's selected rows ----
// rows: the chunk's rows (first4 set); T1, kr1: level-1 threshold bin and the rows of it that
// are selected.  ONE: the one-launch form -- the chunks' counts come from the headers this
// workgroup polls, their lists through agent-scope loads.
template <bool ONE>
DEVI void emit_part(const TopkParams& p, int64_t pair, int c, const ChunkRows& rows, int N, int k, int T1, int kr1) {
    __shared__ int s_hist[kTopkFineBins];
    __shared__ uint32_t s_ckey[SEL_CAP];
    __shared__ int s_cpos[SEL_CAP];
    __shared__ unsigned long long s_sel[SEL_THREADS];   // candidates of this chunk that made the cut
    __shared__ int s_wave[SEL_WAVES + 1];
    __shared__ int s_tot[E_OWN * SEL_WAVES + 1];
    __shared__ int s_pick[2];
    __shared__ uint32_t s_k1[kTopkList];               // the rows of bin T1: keys ...
    __shared__ int s_p1[kTopkList];                    // ... and positions
    __shared__ int s_n1, s_cand, s_before, s_before_eq, s_kr, s_overflow;
    __shared__ uint32_t s_tau;
    __shared__ uint32_t s_hdr[ONE ? kTopkOneMaxChunks : 1];

    const int C = p.chunks;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n4 = (N + 3) >> 2;
    const float* __restrict__ sc = p.scores + pair * p.score_stride;
    const float4* __restrict__ sc4 = reinterpret_cast<const float4*>(sc);
    int32_t* __restrict__ dst = p.idx + pair * (int64_t)p.k;
    if (c == 0)
        for (int i = k + tid; i < p.k; i += SEL_THREADS) dst[i] = -1;  // entries beyond a short sequence
    const int first4 = rows.first4;
    const int chunk_pos0 = 4 * first4, chunk_pos1 = chunk_pos0 + kTopkChunkRows;
    for (int i = tid; i < kTopkFineBins; i += SEL_THREADS) s_hist[i] = 0;
    s_sel[tid] = 0;
    if (tid == 0) s_n1 = 0, s_cand = 0, s_before = 0, s_before_eq = 0, s_overflow = 0, s_pick[0] = SEL_BINS, s_pick[1] = 0;
    if (ONE) {
        // the headers of the pair's chunks, this one's included: one thread each polls (bounded),
        // keeps the value and leaves the unit empty for the next launch
        const int MC = p.max_chunks;
        for (int t = tid; t < C; t += SEL_THREADS) {
            uint64_t* u = p.headers + ((pair * MC + c) * MC + t);
            uint64_t v = 0;
            bool ok = false;
            for (int spin = 0; spin < kTopkHdrSpins && !ok; ++spin) {
                if (spin) __builtin_amdgcn_s_sleep(1);
                v = __hip_atomic_load(u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ok = (uint32_t)(v >> 32) == kTopkHdrFull;
            }
            s_hdr[t] = ok ? (uint32_t)v : 0u;
            __hip_atomic_store(u, (uint64_t)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (!ok && p.err_word) __hip_atomic_store(p.err_word, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
    __syncthreads();
    // every chunk of the pair has read the level-1 histogram (in the first kernel, or -- one
    // launch -- before it sent the header this workgroup now holds): leave it empty
    if (c == 0) *reinterpret_cast<int4*>(p.ghist + pair * SEL_BINS + 4 * tid) = make_int4(0, 0, 0, 0);
    HYLRA_TS_SEL(8);

    // ---- the pair's rows of bin T1 from the chunks' lists into LDS (wave w takes chunks w,
    // w + 16, ...), and the rows above T1 in the chunks before this one ----
    int before = 0;                              // selected rows of the chunks before this one
    for (int cc = wave; cc < C; cc += SEL_WAVES) {
        const int64_t cslot = pair * p.max_chunks + cc;
        const int2 ci = ONE ? make_int2((int)(s_hdr[cc] >> kTopkHdrBits), (int)(s_hdr[cc] & ((1u << kTopkHdrBits) - 1u)))
                            : p.chunk_info[cslot];
        if (ci.y > kTopkChunkList) {
            if (lane == 0) s_overflow = 1;
            continue;
        }
        if (lane == 0 && cc < c) before += ci.x;
        int base = 0;
        if (lane == 0) base = atomicAdd(&s_n1, ci.y);
        base = __shfl(base, 0, 64);
        const int2* __restrict__ gl = p.chunk_list + cslot * kTopkChunkList;
        for (int i = lane; i < ci.y; i += 64) {
            int2 kp;
            if (ONE) {
                const uint64_t e = __hip_atomic_load(reinterpret_cast<const uint64_t*>(gl + i), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                kp = make_int2((int)(uint32_t)e, (int)(uint32_t)(e >> 32));
            } else {
                kp = gl[i];
            }
            if (base + i < kTopkList) {
                s_k1[base + i] = (uint32_t)kp.x;
                s_p1[base + i] = kp.y;
            }
        }
    }
    __syncthreads();
    int n1 = s_n1;
    const bool listed = !s_overflow && n1 <= kTopkList;

    // g(regs, index) for every set of rows of the pair, re-read from memory eight independent
    // loads at a time -- only when the lists do not hold bin T1 (heavy ties)
    auto for_all_rows = [&](auto&& f) {
        constexpr int U = 8;
        for (int i0 = tid; i0 < n4; i0 += U * SEL_THREADS) {
            float4 q[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + u * SEL_THREADS;
                q[u] = i < n4 ? sc4[i] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + u * SEL_THREADS;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (4 * i + e < N) f(4 * i + e, ordered_key(f4_at(q[u], e)));
            }
        }
    };

    // ---- level 2: the rows of bin T1 by their next 12 bits ----
    if (listed) {
        for (int i = tid; i < n1; i += SEL_THREADS) atomicAdd(&s_hist[(s_k1[i] >> 8) & (kTopkFineBins - 1)], 1);
    } else {
        before = 0;
        for_all_rows([&](int pos, uint32_t key) {
            const int b1 = (int)(key >> 20);
            if (b1 > T1) before += pos < chunk_pos0;
            else if (b1 == T1) atomicAdd(&s_hist[(key >> 8) & (kTopkFineBins - 1)], 1);
        });
    }
    __syncthreads();
    HYLRA_TS_SEL(9);
    int h4[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) h4[e] = s_hist[kTopkFineBins - 1 - (4 * tid + e)];
    int T2, above2;
    threshold_pick(h4, kr1, s_wave, s_pick, T2, above2);
    HYLRA_TS_SEL(10);
    const int kr2 = kr1 - above2;                // rows with the top 24 bits (T1, T2) that are selected
    // (T1 = SEL_BINS when nothing is selected: thr24 is then above every 24-bit value)
    const uint32_t thr24 = ((uint32_t)T1 << 12) | (uint32_t)(T2 & (kTopkFineBins - 1));

    // ---- level 3: of the rows of bin T1, those above the 24-bit threshold are selected and those
    // equal to it are candidates ----
    auto classify = [&](int pos, uint32_t key) {
        const uint32_t k24 = key >> 8;
        if (k24 > thr24) {
            before += pos < chunk_pos0;
        } else if (k24 == thr24) {
            const int slot = atomicAdd(&s_cand, 1);
            if (slot < SEL_CAP) {
                s_ckey[slot] = key;
                s_cpos[slot] = pos;
            }
        }
    };
    if (listed) {
        for (int i = tid; i < n1; i += SEL_THREADS) classify(s_p1[i], s_k1[i]);
    } else {
        for_all_rows([&](int pos, uint32_t key) {
            if ((int)(key >> 20) == T1) classify(pos, key);
        });
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) before += __shfl_xor(before, m, 64);
    if (lane == 0 && before) atomicAdd(&s_before, before);
    __syncthreads();
    const int n_cand = s_cand;
    HYLRA_TS_SEL(11);

    unsigned long long sel = 0;                  // bit 4 j + e: element e of own register j is selected
    if (n_cand <= SEL_CAP) {
        // exact rank of every candidate under (key descending, position ascending)
        for (int i = tid; i < n_cand; i += SEL_THREADS) {
            const uint32_t key = s_ckey[i];
            const int pos = s_cpos[i];
            int rank = 0;
            for (int j = 0; j < n_cand; ++j) {
                const uint32_t kj = s_ckey[j];
                rank += (kj > key) || (kj == key && s_cpos[j] < pos);
            }
            if (rank < kr2) {
                if (pos < chunk_pos0) atomicAdd(&s_before, 1);
                else if (pos < chunk_pos1) {
                    const int gl = (pos >> 2) - first4;          // owner thread gl % 1024, register gl / 1024
                    atomicOr(&s_sel[gl & (SEL_THREADS - 1)], 1ull << (4 * (gl >> 10) + (pos & 3)));
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < E_OWN; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (4 * rows.grp(j) + e < N && (rows.key(j, e) >> 8) > thr24) sel |= 1ull << (4 * j + e);
        sel |= s_sel[tid];
    } else {
        // rare: more rows share the top 24 key bits than the candidate list holds (massive
        // ties).  Their last 8 bits decide: histogram, threshold key tau, and of the rows
        // equal to tau the first r in position order.
        __syncthreads();
        for (int i = tid; i < 256; i += SEL_THREADS) s_hist[i] = 0;
        __syncthreads();
        for_all_rows([&](int, uint32_t key) {
            if ((key >> 8) == thr24) atomicAdd(&s_hist[key & 255], 1);
        });
        __syncthreads();
        if (tid == 0) {
            int cnt = 0, dg = 255;
            for (; dg > 0; --dg) {
                if (cnt + s_hist[dg] >= kr2) break;
                cnt += s_hist[dg];
            }
            s_kr = kr2 - cnt;
            s_tau = (thr24 << 8) | (uint32_t)dg;
        }
        __syncthreads();
        const uint32_t tau = s_tau;
        const int r = s_kr;
        // rows before this chunk: above tau inside the 24-bit class, and equal to tau
        int gt_b = 0, eq_b = 0;
        for_all_rows([&](int pos, uint32_t key) {
            if (pos < chunk_pos0 && (key >> 8) == thr24) {
                gt_b += key > tau;
                eq_b += key == tau;
            }
        });
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) {
            gt_b += __shfl_xor(gt_b, m, 64);
            eq_b += __shfl_xor(eq_b, m, 64);
        }
        if (lane == 0) {
            if (gt_b) atomicAdd(&s_before, gt_b);
            if (eq_b) atomicAdd(&s_before_eq, eq_b);
        }
        __syncthreads();
        const int eq_before_chunk = s_before_eq;
        unsigned long long eq_mask = 0;
        int eq_cnt[E_OWN], eq_base[E_OWN];
#pragma unroll
        for (int j = 0; j < E_OWN; ++j) {
            eq_cnt[j] = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (4 * rows.grp(j) + e >= N) continue;
                const uint32_t key = rows.key(j, e);
                if (key > tau) sel |= 1ull << (4 * j + e);
                else if (key == tau) eq_mask |= 1ull << (4 * j + e), ++eq_cnt[j];
            }
        }
        multi_scan<E_OWN>(eq_cnt, eq_base, s_tot);
#pragma unroll
        for (int j = 0; j < E_OWN; ++j) {
            int seen = eq_before_chunk + eq_base[j];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if ((eq_mask >> (4 * j + e)) & 1) {
                    if (seen < r) sel |= 1ull << (4 * j + e);
                    ++seen;
                }
        }
        if (tid == 0) s_before += min(eq_before_chunk, r);
        __syncthreads();
    }
    const int base0 = s_before;
    HYLRA_TS_SEL(12);

    // ---- ordered emission of the chunk's selected rows ----
    int cnt[E_OWN], base[E_OWN];
#pragma unroll
    for (int j = 0; j < E_OWN; ++j) cnt[j] = __popc((unsigned)(sel >> (4 * j)) & 0xFu);
    multi_scan<E_OWN>(cnt, base, s_tot);
#pragma unroll
    for (int j = 0; j < E_OWN; ++j) {
        unsigned nib = (unsigned)(sel >> (4 * j)) & 0xFu;
        int o = base0 + base[j];
        const int pos0 = 4 * rows.grp(j);
        while (nib) {
            const int e = __ffs(nib) - 1;
            nib &= nib - 1;
            if (o < k) dst[o] = pos0 + e;
            ++o;
        }
    }
    HYLRA_TS_SEL(13);
}

// ---- second kernel: levels 2 and 3, ordered emission ----
__global__ __launch_bounds__(SEL_THREADS) void topk_emit_kernel(TopkParams p) {
    int64_t pair;
    int c;
    if (!xcd_pair_role(p.chunks, p.pairs, pair, c)) return;
    const int b = (int)(pair / p.Hkv);
    const int N = seq_units(p.seq_lens, b, p.N, p.sel_block), k = min(p.k, N);
    ChunkRows rows;
    rows.load(p.scores + pair * p.score_stride, (N + 3) >> 2, c);
    const int2 info = p.pair_info[pair];         // level-1 threshold bin; rows in the bins above it
    emit_part<false>(p, pair, c, rows, N, k, info.x, k - info.y);
}

// ---- both in one launch, for launches whose workgroups are all resident at once (the host
// checks).  What crosses workgroups between the two parts -- every chunk's count and list --
// travels as in the Reuse layer's merge by packets: the list with agent-scope stores, and once
// those are acknowledged a 64-bit header {counts, tag} to every chunk of the pair, which the
// receiver polls (bounded), takes and clears.  The chunk's rows stay in registers across the two
// parts, so the scores are read once; one launch and its gap are saved. ----
__global__ __launch_bounds__(SEL_THREADS) void topk_one_kernel(TopkParams p) {
    int64_t pair;
    int c;
    if (!xcd_pair_role(p.chunks + p.merge_wgs, p.pairs, pair, c)) return;
    const int b = (int)(pair / p.Hkv), g = (int)(pair - (int64_t)b * p.Hkv);
    if (merge_part(p, pair, b, g, c)) return;
    const int N = seq_units(p.seq_lens, b, p.N, p.sel_block), k = min(p.k, N);
    ChunkRows rows;
    rows.load(p.scores + pair * p.score_stride, (N + 3) >> 2, c);
    int T1, above1;
    scan_part<true>(p, pair, c, rows, N, k, T1, above1);
    emit_part<true>(p, pair, c, rows, N, k, T1, k - above1);
}

// ---- level-1 histogram in a launch of its own, for the streaming kernels that do not bin ----
// grid (chunks of 8192 rows, Hkv, B); the non-empty bins of a chunk are added to the pair's
// histogram with device-scope atomics.
__global__ __launch_bounds__(SEL_THREADS) void score_hist_kernel(TopkParams p) {
    __shared__ int s_hist[SEL_BINS];
    const int c = blockIdx.x, g = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const int64_t pair = (int64_t)b * p.Hkv + g;
    const int N = seq_units(p.seq_lens, b, p.N, p.sel_block);
    ChunkRows rows;
    rows.load(p.scores + pair * p.score_stride, (N + 3) >> 2, c);
    for (int i = tid; i < SEL_BINS; i += SEL_THREADS) s_hist[i] = 0;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < E_OWN; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (4 * rows.grp(j) + e < N) atomicAdd(&s_hist[rows.key(j, e) >> 20], 1);
    __syncthreads();
    int* gh = p.ghist + pair * SEL_BINS;
    for (int i = tid; i < SEL_BINS; i += SEL_THREADS) {
        const int n = s_hist[i];
        if (n) atomicAdd(gh + i, n);
    }
}

hipError_t launch_score_hist(const TopkParams& p, int B, hipStream_t st) {
    const dim3 grid((p.N + kTopkChunkRows - 1) / kTopkChunkRows, p.Hkv, B);
    hipLaunchKernelGGL(score_hist_kernel, grid, dim3(SEL_THREADS), 0, st, p);
    return hipGetLastError();
}

// chunks, pairs, merge lanes and merge workgroups of a launch
static bool plan_topk(const TopkParams& p, int B, int n_cus, TopkParams& q) {
    q = p;
    q.chunks = p.idx ? (p.N + kTopkChunkRows - 1) / kTopkChunkRows : 0;
    q.pairs = (int64_t)B * p.Hkv;
    if (q.chunks > p.max_chunks) return false;
    // merge of the partials: lanes per output so that a lane has at most four partials (up to 16
    // lanes), workgroups so that one sweep covers the pair's outputs (up to 16 workgroups)
    q.merge_lanes = 1;
    while (q.merge_lanes < 16 && 4 * q.merge_lanes < p.n_splits) q.merge_lanes *= 2;
    q.merge_wgs = (p.G * p.D * q.merge_lanes + SEL_THREADS - 1) / SEL_THREADS;
    if (q.merge_wgs > 16) q.merge_wgs = 16;
    // few partials and already more workgroups than can be resident at once (two per compute
    // unit): the pair's first chunk does the merge in passing
    if (q.chunks > 0 && q.merge_lanes == 1 && q.merge_wgs == 1 && q.pairs * (q.chunks + 1) > 2 * (int64_t)n_cus) q.merge_wgs = 0;
    return true;
}

int topk_one_launch_occupancy() {
    int occ = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, topk_one_kernel, SEL_THREADS, 0) != hipSuccess) return 0;
    return occ;
}

bool topk_one_launch_fits(const TopkParams& p, int B, int n_cus, int occupancy) {
    TopkParams q;
    if (!p.idx || !p.headers || !plan_topk(p, B, n_cus, q)) return false;
    const int64_t wgs = (q.pairs + 7) / 8 * 8 * (q.chunks + q.merge_wgs);
    // (no more workgroups than compute units, although a unit holds `occupancy` of them: that is
    // where one launch wins -- with two workgroups per unit, config 2's 320 and config 4's 512,
    // it only ties with scan + emit -- and it leaves room for whatever else is running)
    return q.chunks >= 1 && q.chunks <= kTopkOneMaxChunks && occupancy >= 1 && wgs <= (int64_t)n_cus;
}

// step 0: scan (+ merge of the partials); step 1: emit; step 2: both in one launch.
// p.idx == nullptr: merge only (step 0).
hipError_t launch_topk(const TopkParams& p, int B, int step, int n_cus, hipStream_t st) {
    TopkParams q;
    if (!plan_topk(p, B, n_cus, q)) return hipErrorInvalidValue;
    if (step == 2 && (!p.headers || q.chunks < 1 || q.chunks > kTopkOneMaxChunks)) return hipErrorInvalidValue;
    const int per_pair = step == 1 ? q.chunks : q.chunks + q.merge_wgs;
    const int64_t wgs = (q.pairs + 7) / 8 * 8 * per_pair;
    if (wgs > 0x7fffffff) return hipErrorInvalidValue;
    if (wgs == 0) return hipSuccess;
    if (step == 0) hipLaunchKernelGGL(topk_scan_kernel, dim3((unsigned)wgs), dim3(SEL_THREADS), 0, st, q);
    else if (step == 1) hipLaunchKernelGGL(topk_emit_kernel, dim3((unsigned)wgs), dim3(SEL_THREADS), 0, st, q);
    else hipLaunchKernelGGL(topk_one_kernel, dim3((unsigned)wgs), dim3(SEL_THREADS), 0, st, q);
    return hipGetLastError();
}

}  // namespace hylra
