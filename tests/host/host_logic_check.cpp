// Host-only check of the library's integer and host-side logic (csrc/host_logic.h), meant to be
// built with g++ -fsanitize=address,undefined and run on the CPU:
//   1. the chunk tables and the claim arithmetic of the self-scheduling Full kernels: for many
//      (tiles, workgroups, sequence length) the chunks of a segment tile its rows exactly once,
//      whichever workgroup claims when, every workgroup ends with exactly one failed claim (none
//      if it never had a chunk to start on), and the claim counter is back at zero afterwards;
//   2. the workgroup-to-group maps (paired_unit, pair_segment) are bijections;
//   3. the policy search against exhaustive search over all policies on small matrices;
//   4. the layout of the Reuse layer's merge packets (every unit has one writer and one reader, a
//      consumer's units are contiguous), the limits under which a launch may merge that way, and
//      the one merge order (blocks of four partials) against a merge in double precision, run
//      through the packets for several launches in a row with the readers clearing what they took.
// The device code reads the tables through the same functions; what is modelled here in plain
// C++ is only the order of the claims (a seeded random interleaving of the workgroups).
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "../../paper_2602_00777_amd/csrc/host_logic.h"

using namespace hylra;

#define CHECK(cond, ...)                                  \
    do {                                                  \
        if (!(cond)) {                                    \
            std::printf("FAILED %s:%d: ", __FILE__, __LINE__); \
            std::printf(__VA_ARGS__);                     \
            std::printf("\n");                            \
            std::exit(1);                                 \
        }                                                 \
    } while (0)

// One workgroup of a segment, as the kernels run it: start on chunk w if there is one (claiming
// at once if that chunk is empty), then claim until the counter has run out.
struct Wg {
    int w;
    bool started = false, done = false;
    int failed_claims = 0;
};

static void claim(const int* table, const SegInfo& sg, int& ctr, int& adds, std::vector<int>& cover, Wg& g) {
    // settle_claim: claims until a chunk has tiles or the counter runs out; the claim that draws
    // the last value stores zero
    for (;;) {
        const int raw = ctr++;
        ++adds;
        if (raw == sg.n_eff - 1) ctr = 0;
        const int c = sg.wgs + raw;
        if (c >= sg.n_eff) {
            ++g.failed_claims;
            g.done = true;
            return;
        }
        const int lo = chunk_bound(table, sg, c), hi = chunk_bound(table, sg, c + 1);
        if (hi > lo) {
            for (int t = lo; t < hi; ++t) ++cover[t];
            return;
        }
    }
}

static void check_segment(int made_for, int S, int tiles, int wgs, std::mt19937& rng) {
    int table[kMaxChunks + 1];
    const int n_chunks = make_chunk_table(made_for, S, table);
    CHECK(n_chunks >= 1 && n_chunks <= kMaxChunks && table[0] == 0 && table[n_chunks] == made_for, "table ends");
    for (int c = 0; c < n_chunks; ++c) CHECK(table[c + 1] > table[c], "chunk %d is empty in the table", c);
    SegInfo sg{};
    sg.tile0 = 0, sg.tiles = tiles, sg.made_for = made_for, sg.wgs = wgs;
    seg_chunks(table, n_chunks, sg);
    CHECK(sg.n_eff >= 1 && sg.c0 + sg.n_eff == n_chunks, "n_eff");
    CHECK(chunk_bound(table, sg, 0) == 0 && chunk_bound(table, sg, sg.n_eff) == tiles, "segment ends");
    std::vector<int> cover(tiles, 0);
    std::vector<Wg> g(wgs);
    int ctr = 0, adds = 0;
    for (int w = 0; w < wgs; ++w) g[w].w = w;
    // random interleaving: pick a workgroup that is not done and let it take its next step
    std::vector<int> alive(wgs);
    for (int w = 0; w < wgs; ++w) alive[w] = w;
    while (!alive.empty()) {
        const size_t pick = rng() % alive.size();
        Wg& x = g[alive[pick]];
        if (!x.started) {
            x.started = true;
            if (x.w < sg.n_eff) {
                const int lo = chunk_bound(table, sg, x.w), hi = chunk_bound(table, sg, x.w + 1);
                if (hi > lo) {
                    for (int t = lo; t < hi; ++t) ++cover[t];
                } else {
                    claim(table, sg, ctr, adds, cover, x);
                }
            } else {
                x.done = true;          // more workgroups than chunks: neither starts nor claims
            }
        } else {
            claim(table, sg, ctr, adds, cover, x);
        }
        if (x.done) {
            alive[pick] = alive.back();
            alive.pop_back();
        }
    }
    for (int t = 0; t < tiles; ++t) CHECK(cover[t] == 1, "tile %d of %d covered %d times (made_for %d S %d wgs %d)", t, tiles, cover[t], made_for, S, wgs);
    CHECK(ctr == 0, "counter is %d after the launch (made_for %d S %d tiles %d wgs %d)", ctr, made_for, S, tiles, wgs);
    CHECK(adds == sg.n_eff, "%d claims for %d chunks (wgs %d)", adds, sg.n_eff, wgs);
    for (const Wg& x : g) CHECK(x.failed_claims == (x.w < sg.n_eff ? 1 : 0), "workgroup %d: %d failed claims", x.w, x.failed_claims);
}

static void check_maps() {
    for (int S : {2, 4, 8, 16})
        for (int units : {1, 2, 3, 8, 64}) {
            const int half = units * S / 2;
            std::vector<int> seen(2 * half, 0);
            for (int x = 0; x < 2 * half; ++x) {
                int unit, w;
                paired_unit(x, half, S, unit, w);
                CHECK(unit >= 0 && unit < units && w >= 0 && w < S, "paired_unit range");
                ++seen[unit * S + w];
            }
            for (int v : seen) CHECK(v == 1, "paired_unit is not a bijection (S %d units %d)", S, units);
        }
    for (int S : {1, 2, 3, 8})
        for (int n = 1; n <= 50; ++n) {
            int next_wg0 = 0, last_seg = -1;
            for (int w = 0; w < n; ++w) {
                const PairSeg ps = pair_segment(n, S, w);
                CHECK(ps.w >= 0 && ps.w < ps.wgs && ps.wg0 + ps.w == w, "pair_segment rank");
                if (ps.seg != last_seg) {
                    CHECK(ps.seg == last_seg + 1 && ps.wg0 == next_wg0 && ps.w == 0, "pair_segment order");
                    next_wg0 += ps.wgs;
                    last_seg = ps.seg;
                }
                if (n >= S) CHECK(ps.wgs >= S && ps.wgs <= 2 * S - 1, "segment of %d workgroups (n %d S %d)", ps.wgs, n, S);
            }
            CHECK(next_wg0 == n, "segments do not add up");
        }
}

static void check_policy(std::mt19937& rng) {
    std::uniform_real_distribution<double> u(0.0, 1.0);
    for (int rep = 0; rep < 200; ++rep) {
        const int L = 1 + (int)(rng() % 9);
        std::vector<double> M((size_t)L * L, 0.0);
        const bool coarse = rep % 2;            // quantised entries: many ties
        for (int i = 0; i < L; ++i)
            for (int j = i; j < L; ++j) M[(size_t)i * L + j] = i == j ? 1.0 : coarse ? (double)(rng() % 4) / 4.0 : u(rng);
        const double theta = coarse ? 0.5 : u(rng);
        std::vector<uint8_t> pol(L);
        double s = 0.0;
        const int c = policy_search_host(L, M.data(), theta, pol.data(), &s);
        // the returned policy is feasible and has the value it claims
        CHECK(pol[0] == 0, "layer 0 must be Full");
        int full = 0, src = 0;
        double sim = 0.0;
        for (int j = 0; j < L; ++j) {
            if (pol[j] == 0) src = j, ++full;
            else CHECK(M[(size_t)src * L + j] >= theta, "reuse below the threshold");
            sim += M[(size_t)src * L + j];
        }
        CHECK(full == c && sim > s - 1e-9 && sim < s + 1e-9, "value of the policy");
        // no policy is better (fewer Full layers, then a larger sum)
        for (unsigned mask = 0; mask < (1u << (L - 1)); ++mask) {
            int f = 1, sr = 0;
            double sm = M[0];
            bool ok = true;
            for (int j = 1; j < L && ok; ++j) {
                if (!((mask >> (j - 1)) & 1)) sr = j, ++f;
                else ok = M[(size_t)sr * L + j] >= theta;
                sm += M[(size_t)sr * L + j];
            }
            if (ok) CHECK(f > c || (f == c && sm <= s + 1e-9), "a better policy exists");
        }
        std::vector<int64_t> counts((size_t)L * L, 0);
        for (int i = 0; i < L; ++i)
            for (int j = i; j < L; ++j) counts[(size_t)i * L + j] = i == j ? 10 + j : (int64_t)(rng() % 10);
        std::vector<double> Ms((size_t)L * L, -1.0);
        similarity_from_counts(L, counts.data(), Ms.data());
        for (int i = 0; i < L; ++i)
            for (int j = 0; j < L; ++j) {
                const double want = i > j ? 0.0 : i == j ? 1.0 : (double)counts[(size_t)i * L + j] / (double)counts[(size_t)j * L + j];
                CHECK(Ms[(size_t)i * L + j] == want, "similarity matrix");
            }
    }
}

// Packets: the producers' unit numbers (as send_packets forms them) against the consumers'
// (consumer c polls units [c S PK, (c + 1) S PK) and finds partial s's head-h values at
// s PK + 2 h, + 1 and its element (h, j) at s PK + 2 G + h W + j of that range), over several
// launches on one buffer that starts all empty and that the readers clear.
static void check_packets(std::mt19937& rng) {
    const int D = 128;
    std::uniform_real_distribution<float> val(-3.f, 3.f), pos(0.1f, 50.f);
    for (int G = 1; G <= 8; ++G)
        for (int S : {4, 8, 16, 32, 64, 128}) {
            const PacketShape ps = packet_shape(G, D, S);
            CHECK(ps.W * S == D && ps.PK == G * (2 + ps.W), "shape G=%d S=%d", G, S);
            const int64_t total = (int64_t)S * S * ps.PK;
            std::vector<uint64_t> buf(total, 0);                 // {value, tag} units, tag 0 = empty
            for (int launch = 0; launch < 3; ++launch) {
                std::vector<float> m(S * G), l(S * G), acc((size_t)S * G * D);
                for (auto& x : m) x = val(rng);
                for (auto& x : l) x = pos(rng);
                for (auto& x : acc) x = val(rng);
                if (launch == 1)                                  // a producer that saw no rows
                    for (int h = 0; h < G; ++h) m[h] = -1.0e30f, l[h] = 0.f;
                auto put = [&](int64_t u, float v) {
                    CHECK(u >= 0 && u < total, "unit %lld outside the pair's %lld", (long long)u, (long long)total);
                    CHECK((buf[u] >> 32) == 0, "unit %lld written twice (G=%d S=%d)", (long long)u, G, S);
                    uint32_t bits;
                    std::memcpy(&bits, &v, 4);
                    buf[u] = ((uint64_t)1 << 32) | bits;
                };
                for (int s = 0; s < S; ++s) {
                    for (int h = 0; h < G; ++h)
                        for (int col = 0; col < D; ++col) put(packet_acc_unit(ps, G, s, h, col), acc[((size_t)s * G + h) * D + col]);
                    for (int c = 0; c < S; ++c)
                        for (int h = 0; h < G; ++h) {
                            put(packet_ml_unit(ps, c, s, h, 0), m[s * G + h]);
                            put(packet_ml_unit(ps, c, s, h, 1), l[s * G + h]);
                        }
                }
                for (int64_t u = 0; u < total; ++u) CHECK((buf[u] >> 32) == 1, "unit %lld never written (G=%d S=%d)", (long long)u, G, S);
                for (int c = 0; c < S; ++c) {
                    const int64_t first = packet_ml_unit(ps, c, 0, 0, 0);
                    CHECK(first == (int64_t)c * S * ps.PK, "consumer %d starts at %lld", c, (long long)first);
                    std::vector<float> pk((size_t)S * ps.PK);
                    for (int i = 0; i < S * ps.PK; ++i) {
                        const uint32_t bits = (uint32_t)buf[first + i];
                        std::memcpy(&pk[i], &bits, 4);
                        buf[first + i] = 0;                       // the reader clears what it took
                    }
                    for (int h = 0; h < G; ++h)
                        for (int j = 0; j < ps.W; ++j) {
                            float M = -1.0e30f;
                            for (int s = 0; s < S; ++s) M = std::fmax(M, pk[s * ps.PK + 2 * h]);
                            // as the consumer's lanes do it: one block of four per lane, block sums in block order
                            float den = 0.f, num = 0.f;
                            for (int blk = 0; blk < S / kMergeBlock; ++blk) {
                                float db = 0.f, nb = 0.f;
                                for (int i = 0; i < kMergeBlock; ++i) {
                                    const int s = blk * kMergeBlock + i;
                                    const float w = std::exp2(pk[s * ps.PK + 2 * h] - M);
                                    db = std::fmaf(w, pk[s * ps.PK + 2 * h + 1], db);
                                    nb = std::fmaf(w, pk[s * ps.PK + 2 * G + h * ps.W + j], nb);
                                }
                                den += db, num += nb;
                            }
                            const float got = den > 0.f ? num / den : 0.f;
                            // the sequential form of the same order, fed straight from the producers' values
                            MergeSum sum;
                            double dn = 0.0, dd = 0.0;
                            const int col = c * ps.W + j;
                            for (int s = 0; s < S; ++s) {
                                const float w = std::exp2(m[s * G + h] - M);
                                sum.add(s, w, l[s * G + h], acc[((size_t)s * G + h) * D + col]);
                                dn += (double)w * acc[((size_t)s * G + h) * D + col];
                                dd += (double)w * l[s * G + h];
                            }
                            const float want = sum.result();
                            CHECK(std::memcmp(&got, &want, 4) == 0 || (got == 0.f && want == 0.f), "merge order differs: %g vs %g (G=%d S=%d)", got, want, G, S);
                            CHECK(std::fabs(got - dn / dd) <= 1e-5 * (1.0 + std::fabs(dn / dd)), "merge value %g vs %g", got, dn / dd);
                        }
                }
                for (int64_t u = 0; u < total; ++u) CHECK(buf[u] == 0, "unit %lld left full after the launch", (long long)u);
            }
        }
    // the limits: what the benchmark shapes choose, and what must be refused
    const int64_t cap = 256 * 6 * 512;
    CHECK(packets_fit(8, 32, 4, 128, 256, 6, 256, cap, 8), "batch 1, 8 KV heads, k = 4096");
    CHECK(packets_fit(16, 16, 7, 128, 256, 6, 256, cap, 8), "batch 4, 4 KV heads of 7, k = 2048");
    CHECK(packets_fit(2, 32, 8, 128, 256, 6, 256, cap, 8), "G = 8 with 32 partials just fits 6 units per thread");
    CHECK(!packets_fit(1, 64, 8, 128, 256, 6, 256, cap, 8), "G = 8 with 64 partials: more than a thread polls");
    CHECK(!packets_fit(64, 4, 4, 128, 512, 6, 256, cap, 8), "4 partials: below the automatic minimum");
    CHECK(packets_fit(64, 4, 4, 128, 512, 6, 256, cap, 4), "4 partials when asked for");
    CHECK(!packets_fit(64, 8, 4, 128, 256, 6, 256, cap, 8), "more workgroups than compute units");
    CHECK(!packets_fit(8, 24, 4, 128, 256, 6, 256, cap, 8) && !packets_fit(8, 2, 4, 128, 256, 6, 256, cap, 2) && !packets_fit(1, 256, 1, 128, 256, 6, 256, cap, 8),
          "not a power of two, fewer than a merge block, more partials than columns");
    CHECK(!packets_fit(8, 32, 4, 128, 256, 6, 256, 1000, 8), "buffer too small");
}

int main() {
    std::mt19937 rng(12345);
    int cases = 0;
    for (int S : {1, 2, 3, 4, 8})
        for (int made_for : {1, 3, 4, 17, 128, 1024, 4099, 65536}) {
            for (int rep = 0; rep < 6; ++rep) {
                // a full-length sequence has made_for or made_for + 1 tiles; shorter ones any number
                const int tiles = rep == 0 ? made_for : rep == 1 ? made_for + 1 : 1 + (int)(rng() % made_for);
                for (int wgs : {S, S + 1, 2 * S - 1 > 0 ? 2 * S - 1 : 1, 1, 40}) {
                    check_segment(made_for, S, tiles, wgs, rng);
                    ++cases;
                }
            }
        }
    check_maps();
    check_policy(rng);
    check_packets(rng);
    std::printf("host logic ok: %d segment cases\n", cases);
    return 0;
}
