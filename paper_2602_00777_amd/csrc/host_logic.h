// The library's integer and host-side logic that needs no GPU: the chunk tables and segment
// arithmetic of the self-scheduling Full kernels (used on the host to build the tables and on
// the device to read them), the workgroup-to-group maps, and the offline policy search
// (Algorithm 1; similarity matrix as in Eq. 2).  Plain C++ with no HIP types, so that it also
// compiles with the host compiler alone: tests/host_logic_check.cpp runs it under the address
// and undefined-behaviour sanitizers.
#pragma once
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
