// The library's integer and host-side logic that needs no GPU: the chunk tables and segment
// arithmetic of the self-scheduling Full kernels (used on the host to build the tables and on
// the device to read them), the workgroup-to-group maps, the layout of the Reuse layer's merge
// packets, and the offline policy search (Algorithm 1; similarity matrix as in Eq. 2).  Plain C++ with no HIP types, so that it also
// compiles with the host compiler alone: tests/host_logic_check.cpp runs it under the address
// and undefined-behaviour sanitizers.
#pragma once
#include <math.h>
#include <stdint.h>

#include <vector>

#if defined(__HIPCC__)
#define HYLRA_HD __host__ __device__ __forceinline__
#else
#define HYLRA_HD inline
#endif

namespace hylra {

constexpr int kMaxChunks = 480;     // chunks of rows per (batch, KV head) in the self-scheduling Full kernel

HYLRA_HD int64_t ceil_div64(int64_t x, int64_t m) { return (x + m - 1) / m; }

// ---- chunk table (guided self-scheduling) --------------------------------------------------
// With `remaining` tiles left, the next chunk takes remaining / (2 * S) of them, never fewer than
// min_tiles (one tile per wave; doubled until the table fits), so chunks shrink towards the end
// and the S workgroups of a (batch, KV head) finish within about one small chunk of each other.
// chunk_tile[c] = first tile of chunk c, chunk_tile[n] = total_tiles.  Returns n.
inline int make_chunk_table(int total_tiles, int S, int (&chunk_tile)[kMaxChunks + 1]) {
    for (int min_tiles = 4;; min_tiles *= 2) {
        int n = 0, at = 0;
        while (at < total_tiles && n < kMaxChunks) {
            int take = (int)ceil_div64(total_tiles - at, 2 * (int64_t)S);
            if (take < min_tiles) take = min_tiles;
            if (take > total_tiles - at) take = total_tiles - at;
            chunk_tile[n++] = at;
            at += take;
        }
        if (at == total_tiles) {
            chunk_tile[n] = total_tiles;
            return n;
        }
    }
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

HYLRA_HD void seg_chunks(const int* chunk_tile, int n_chunks, SegInfo& sg) {
    sg.off = sg.made_for - sg.tiles > 0 ? sg.made_for - sg.tiles : 0;
    int lo = 0, hi = sg.off ? n_chunks : 0;         // largest c with chunk_tile[c] <= off (0 for a full-length sequence)
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (chunk_tile[mid] <= sg.off) lo = mid;
        else hi = mid - 1;
    }
    sg.c0 = lo;
    sg.n_eff = n_chunks - lo;
}

// First tile (within the segment) of the segment's chunk c (0 .. n_eff - 1); chunk c is
// [chunk_bound(c), chunk_bound(c + 1)).
HYLRA_HD int chunk_bound(const int* chunk_tile, const SegInfo& sg, int c) {
    if (c >= sg.n_eff) return sg.tiles;
    const int t = chunk_tile[sg.c0 + c] - sg.off;
    return t > 0 ? t : 0;
}

// Workgroup x of a grid of 2 * half workgroups -> the group of S workgroups (S even) it belongs
// to and its rank there: group u is made of the S / 2 workgroups u * S / 2 .. of the first half
// and of the S / 2 workgroups of the second half that sit one group further on (so that its
// workgroups of the second half land on other XCDs than those of the first half).
HYLRA_HD void paired_unit(int x, int half, int S, int& unit, int& w) {
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
HYLRA_HD PairSeg pair_segment(int n, int S, int w) {
    const int n_seg = n / S > 1 ? n / S : 1, base = n / n_seg, extra = n - base * n_seg;   // `extra` segments have one more
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

// ---- the one merge order ---------------------------------------------------------------------
constexpr int kMergeBlock = 4;      // partials per block
// Merge of S online-softmax partials (max m_s in log2 units, sum l_s, accumulator a_s) into
// out = sum_s w_s a_s / sum_s w_s l_s with w_s = 2^(m_s - max m).  Every merge in this library
// adds in ONE order, so that they agree bit for bit whichever kernel runs it: blocks of four
// consecutive partials are accumulated from zero with fused multiply-adds, and the block sums
// are added to the total in block order (a lane per block can then share one element's merge).
struct MergeSum {
    float num = 0.f, den = 0.f;     // totals
    float nb = 0.f, db = 0.f;       // the block under way
    HYLRA_HD void add(int s, float w, float l, float a) {       // s = 0, 1, 2, ... in order
        if (s % kMergeBlock == 0 && s) close_block();
        db = fmaf(w, l, db);
        nb = fmaf(w, a, nb);
    }
    HYLRA_HD void close_block() {
        num += nb, den += db;
        nb = 0.f, db = 0.f;
    }
    HYLRA_HD float result() {
        close_block();
        return den > 0.f ? num / den : 0.f;
    }
};

// ---- merge by packets (Reuse layer): layout and limits ---------------------------------------
// The S workgroups of a (batch, KV head) each merge D / S output columns of all G heads.
// Producer s sends consumer c one packet of G (2 + D / S) units: [G][2] (max, sum) and then
// [G][D / S] (its accumulator's columns c D / S ..).  The packets of a pair are laid out
// [consumer][producer][unit], so that what a consumer polls is contiguous.
struct PacketShape {
    int S, W, PK;                   // partials per pair, columns per consumer, units per packet
};
HYLRA_HD PacketShape packet_shape(int G, int D, int S) {
    PacketShape ps;
    ps.S = S, ps.W = D / S, ps.PK = G * (2 + D / S);
    return ps;
}
// unit (within the pair's S * S * PK) of head h's max (which = 0) or sum (1) from producer s to consumer c
HYLRA_HD int64_t packet_ml_unit(const PacketShape& ps, int c, int s, int h, int which) {
    return ((int64_t)c * ps.S + s) * ps.PK + 2 * h + which;
}
// unit of accumulator element (h, col) of producer s; G: heads per pair
HYLRA_HD int64_t packet_acc_unit(const PacketShape& ps, int G, int s, int h, int col) {
    const int c = col / ps.W, j = col - c * ps.W;
    return ((int64_t)c * ps.S + s) * ps.PK + 2 * G + h * ps.W + j;
}
// Whether a launch of `pairs` pairs with n partials each may merge by packets: every workgroup
// resident at once (at most one per compute unit), n a power of two between min_n and D (so
// that it divides the D columns and groups of n / 4 lanes line up), what a workgroup of
// `threads` threads receives within units_per_thread units per thread, everything within the
// buffer of cap_units units.
HYLRA_HD bool packets_fit(int64_t pairs, int64_t n, int G, int D, int threads, int units_per_thread, int n_cus,
                          int64_t cap_units, int min_n) {
    if (n < min_n || n < 4 || n > D || (n & (n - 1)) != 0 || D % n != 0) return false;
    const int64_t per_consumer = n * (int64_t)G * (2 + D / n);
    return pairs * n <= n_cus && per_consumer <= (int64_t)units_per_thread * threads && pairs * n * per_consumer <= cap_units;
}

// ---- offline profiling (host only) -----------------------------------------------------------
// M[i][j] = counts[i][j] / counts[j][j] for i <= j (diagonal 1; a layer without valid entries
// gets 0 off the diagonal), 0 below the diagonal.
inline void similarity_from_counts(int L, const int64_t* counts, double* M) {
    for (int64_t i = 0; i < L; ++i)
        for (int64_t j = 0; j < L; ++j) {
            const int64_t d = counts[j * L + j];
            M[i * L + j] = i > j ? 0.0 : i == j ? 1.0 : d > 0 ? (double)counts[i * L + j] / (double)d : 0.0;
        }
}

// Algorithm 1.  A state (i, j), i <= j: layer j uses the index set of layer i (i == j: full
// attention at layer j).  Layer by layer, every state keeps the best value of a path that
// reaches it: fewest Full layers first, then the largest sum of similarities; a later candidate
// replaces it only if strictly better (candidates arrive in the order of the algorithm's
// loops).  Returns the number of Full layers of the best path.
inline int policy_search_host(int L, const double* M, double theta, uint8_t* policy, double* sum_sim) {
    struct Val {
        int full = -1;          // -1: not reachable
        double sim = 0.0;
        int from = -1;          // source layer of the state this one was reached from
        bool better_than(const Val& o) const { return o.full < 0 || full < o.full || (full == o.full && sim > o.sim); }
    };
    // column j of the state grid: states (0..j, j)
    std::vector<std::vector<Val>> col(L);
    col[0].resize(1);
    col[0][0].full = 1, col[0][0].sim = M[0];
    for (int j = 1; j < L; ++j) {
        col[j].resize(j + 1);
        const double diag = M[(size_t)j * L + j];
        for (int i = 0; i < j; ++i) {
            const Val& v = col[j - 1][i];
            if (v.full < 0) continue;
            const double m = M[(size_t)i * L + j];
            if (m >= theta) {                               // index reuse: (i, j-1) -> (i, j)
                Val c;
                c.full = v.full, c.sim = v.sim + m, c.from = i;
                if (c.better_than(col[j][i])) col[j][i] = c;
            }
            Val c;                                          // full attention: (i, j-1) -> (j, j)
            c.full = v.full + 1, c.sim = v.sim + diag, c.from = i;
            if (c.better_than(col[j][j])) col[j][j] = c;
        }
    }
    int best = -1;
    for (int i = 0; i < L; ++i)
        if (col[L - 1][i].full >= 0 && (best < 0 || col[L - 1][i].better_than(col[L - 1][best]))) best = i;
    if (sum_sim) *sum_sim = col[L - 1][best].sim;
    const int n_full = col[L - 1][best].full;
    for (int j = L - 1, i = best; j >= 0; --j) {
        policy[j] = i == j ? 0 : 1;
        i = col[j][i].from;
    }
    return n_full;
}

}  // namespace hylra
