/*
 * CPU oracle for the HyLRA per-layer decode-attention step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP path is checked against.  It shares no code, header, table or helper
 * with the GPU library and must never be called from the product path.
 *
 * What it computes (paper: Eq. 1 in "Intra-Layer Sensitivity"; Algorithm 2
 * "Hybrid Inter-Layer Top-K Reuse Attention"):
 *
 *   Full layer   S = Score(Q, K^cache) = Q K^T / sqrt(d)          (Alg. 2, Full branch; Eq. 1)
 *                I = TopK(S, budget)                               (Alg. 2, Full branch)
 *                O = Softmax(S) V^cache   over ALL N rows          (Alg. 2, Full branch)
 *   Reuse layer  I inherited unchanged from the previous layer     (Alg. 2, Reuse branch)
 *                O = Attention(Q, K^cache[I], V^cache[I])          (Alg. 2, Reuse branch; Eq. 1)
 *   Step         layers visited in order, policy decides the branch (Alg. 2 outer loop)
 *
 * Readings the paper leaves open (the algorithm is stated for one head):
 *   - several query heads share one KV head (grouped-query attention): query
 *     head h reads KV head h / G, G = Hq / Hkv; ONE index set per (batch, KV
 *     head), ranked by the MEAN over the G heads of the scaled logits;
 *   - ties in the ranking go to the lower position; the k positions are
 *     returned in ascending order;
 *   - negative entries in an inherited index set are padding and are skipped.
 *
 * Arithmetic: everything in double.  Inputs arrive either as doubles or as
 * bf16 bit patterns (uint16, upper half of an IEEE binary32), which convert to
 * double exactly.  No blocking, no online softmax, no fusion: scores for all N
 * rows are materialised, the maximum is subtracted, weights are normalised by
 * their plain sum.
 *
 * Layouts (all contiguous, row-major):
 *   q   [B, Hq, d]        K, V [B, Hkv, N, d]
 *   out [B, Hq, d] double idx  [B, Hkv, k] int32     shat [B, Hkv, N] double
 *
 * Also here, for the offline profiling step that produces the policy (Eq. 2, Algorithm 1):
 * the pooled overlap counts between the layers' index sets and the policy search.
 *
 * Parity pins for every function here live in tests/test_oracle_pins.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F64 = 0, ORACLE_BF16 = 1 };

enum {
    ORACLE_OK = 0,
    ORACLE_BAD_ARG = 1,
    ORACLE_POLICY = 4,
    ORACLE_NOMEM = 6
};

/* element i of a tensor stored either as double or as bf16 bit patterns */
static double elem(const void *base, int kind, size_t i)
{
    if (kind == ORACLE_F64)
        return ((const double *)base)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static int shape_ok(int B, int Hq, int Hkv, int d, long N)
{
    return B > 0 && Hq > 0 && Hkv > 0 && d > 0 && N > 0 && Hq % Hkv == 0;
}

typedef struct {
    double score;
    int32_t pos;
} ranked;

/* descending score, then ascending position */
static int by_score_then_pos(const void *a, const void *b)
{
    const ranked *x = a, *y = b;
    if (x->score > y->score) return -1;
    if (x->score < y->score) return 1;
    return (x->pos > y->pos) - (x->pos < y->pos);
}

static int by_pos(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* s[j] = scale * <q_h, K_j>, j = 0..N-1          (Alg. 2 "Score"; Eq. 1) */
static void score_rows(const void *q, const void *K, int kind, size_t q_off,
                       size_t k_off, int d, long N, double scale, double *s)
{
    for (long j = 0; j < N; ++j) {
        double dot = 0.0;
        for (int c = 0; c < d; ++c)
            dot += elem(q, kind, q_off + c) * elem(K, kind, k_off + (size_t)j * d + c);
        s[j] = scale * dot;
    }
}

/*
 * Full layer.  out may be NULL (skip the output), idx may be NULL (skip the
 * selection), shat may be NULL.  scale <= 0 means 1/sqrt(d).
 */
int hylra_oracle_full_attn_topk(int kind, int B, int Hq, int Hkv, int d, long N, int k,
                                double scale, const void *q, const void *K, const void *V,
                                double *out, int32_t *idx, double *shat)
{
    if (!shape_ok(B, Hq, Hkv, d, N) || !q || !K || !V) return ORACLE_BAD_ARG;
    if (idx && (k < 1 || k > N)) return ORACLE_BAD_ARG;
    if (kind != ORACLE_F64 && kind != ORACLE_BF16) return ORACLE_BAD_ARG;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)d);
    const int G = Hq / Hkv;
    int failed = 0;

#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        for (int g = 0; g < Hkv; ++g) {
            double *s = malloc((size_t)N * sizeof *s);
            double *mean = calloc((size_t)N, sizeof *mean);
            double *w = malloc((size_t)N * sizeof *w);
            ranked *r = malloc((size_t)N * sizeof *r);
            if (!s || !mean || !w || !r) {
#pragma omp atomic write
                failed = 1;
                free(s); free(mean); free(w); free(r);
                continue;
            }
            const size_t kv_off = ((size_t)b * Hkv + g) * (size_t)N * d;

            for (int hh = 0; hh < G; ++hh) {
                const int h = g * G + hh;            /* heads of one group are consecutive */
                const size_t q_off = ((size_t)b * Hq + h) * d;
                score_rows(q, K, kind, q_off, kv_off, d, N, scale, s);
                for (long j = 0; j < N; ++j) mean[j] += s[j];

                if (out) {                            /* O = Softmax(S) V, dense over all N */
                    double m = s[0];
                    for (long j = 1; j < N; ++j) if (s[j] > m) m = s[j];
                    double z = 0.0;
                    for (long j = 0; j < N; ++j) { w[j] = exp(s[j] - m); z += w[j]; }
                    for (int c = 0; c < d; ++c) {
                        double acc = 0.0;
                        for (long j = 0; j < N; ++j)
                            acc += w[j] * elem(V, kind, kv_off + (size_t)j * d + c);
                        out[q_off + c] = acc / z;
                    }
                }
            }
            for (long j = 0; j < N; ++j) mean[j] /= (double)G;
            if (shat)
                memcpy(shat + ((size_t)b * Hkv + g) * (size_t)N, mean, (size_t)N * sizeof *mean);

            if (idx) {                                /* I = TopK(mean score, k) */
                for (long j = 0; j < N; ++j) { r[j].score = mean[j]; r[j].pos = (int32_t)j; }
                qsort(r, (size_t)N, sizeof *r, by_score_then_pos);
                int32_t *dst = idx + ((size_t)b * Hkv + g) * (size_t)k;
                for (int t = 0; t < k; ++t) dst[t] = r[t].pos;
                qsort(dst, (size_t)k, sizeof *dst, by_pos);
            }
            free(s); free(mean); free(w); free(r);
        }
    }
    return failed ? ORACLE_NOMEM : ORACLE_OK;
}

/*
 * Reuse layer: attention restricted to the rows named by idx[b, g, 0..k-1].
 * Negative entries are skipped; entries >= N are an error.  If a set has no
 * valid entry the output row is zero.
 */
int hylra_oracle_reuse_sparse_attn(int kind, int B, int Hq, int Hkv, int d, long N, int k,
                                   double scale, const void *q, const void *K, const void *V,
                                   const int32_t *idx, double *out)
{
    if (!shape_ok(B, Hq, Hkv, d, N) || !q || !K || !V || !idx || !out || k < 1)
        return ORACLE_BAD_ARG;
    if (kind != ORACLE_F64 && kind != ORACLE_BF16) return ORACLE_BAD_ARG;
    for (size_t t = 0; t < (size_t)B * Hkv * k; ++t)
        if (idx[t] >= N) return ORACLE_BAD_ARG;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)d);
    const int G = Hq / Hkv;
    int failed = 0;

#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < Hq; ++h) {
            const int g = h / G;
            const int32_t *T = idx + ((size_t)b * Hkv + g) * (size_t)k;
            const size_t kv_off = ((size_t)b * Hkv + g) * (size_t)N * d;
            const size_t q_off = ((size_t)b * Hq + h) * d;
            double *s = malloc((size_t)k * sizeof *s);
            if (!s) {
#pragma omp atomic write
                failed = 1;
                continue;
            }
            /* scores of the gathered rows: K^sparse = K^cache[I] */
            int any = 0;
            double m = 0.0;
            for (int t = 0; t < k; ++t) {
                if (T[t] < 0) continue;
                double dot = 0.0;
                for (int c = 0; c < d; ++c)
                    dot += elem(q, kind, q_off + c) * elem(K, kind, kv_off + (size_t)T[t] * d + c);
                s[t] = scale * dot;
                if (!any || s[t] > m) m = s[t];
                any = 1;
            }
            double z = 0.0;
            for (int t = 0; t < k; ++t)
                if (T[t] >= 0) { s[t] = exp(s[t] - m); z += s[t]; }
            for (int c = 0; c < d; ++c) {
                double acc = 0.0;
                for (int t = 0; t < k; ++t)
                    if (T[t] >= 0)
                        acc += s[t] * elem(V, kind, kv_off + (size_t)T[t] * d + c);
                out[q_off + c] = any ? acc / z : 0.0;
            }
            free(s);
        }
    }
    return failed ? ORACLE_NOMEM : ORACLE_OK;
}

/*
 * One decode step over L layers (Alg. 2 outer loop).  policy[l] = 0 is Full,
 * 1 is Reuse; policy[0] must be Full (there is nothing to inherit before it).
 * q_l, K_l, V_l, out_l are arrays of L pointers.  idx_cur [B, Hkv, k] holds,
 * on return, the set chosen by the last Full layer.  If idx_trace is not NULL
 * it receives the set in force at every layer, [L, B, Hkv, k].
 */
int hylra_oracle_decode_step(int kind, int L, const uint8_t *policy, int B, int Hq, int Hkv,
                             int d, long N, int k, double scale, const void *const *q_l,
                             const void *const *K_l, const void *const *V_l,
                             double *const *out_l, int32_t *idx_cur, int32_t *idx_trace)
{
    if (L < 1 || !policy || !q_l || !K_l || !V_l || !out_l || !idx_cur) return ORACLE_BAD_ARG;
    if (policy[0] != 0) return ORACLE_POLICY;
    for (int l = 0; l < L; ++l)
        if (policy[l] > 1) return ORACLE_POLICY;
    const size_t set = (size_t)B * Hkv * k;
    for (int l = 0; l < L; ++l) {
        int rc;
        if (policy[l] == 0)
            rc = hylra_oracle_full_attn_topk(kind, B, Hq, Hkv, d, N, k, scale, q_l[l], K_l[l],
                                             V_l[l], out_l[l], idx_cur, NULL);
        else    /* I_l <- I_{l-1}: idx_cur is simply left as it is */
            rc = hylra_oracle_reuse_sparse_attn(kind, B, Hq, Hkv, d, N, k, scale, q_l[l],
                                                K_l[l], V_l[l], idx_cur, out_l[l]);
        if (rc != ORACLE_OK) return rc;
        if (idx_trace) memcpy(idx_trace + (size_t)l * set, idx_cur, set * sizeof *idx_cur);
    }
    return ORACLE_OK;
}

/*
 * Block-level variant (paper, "Adaptation to block-level sparsity"): consecutive tokens are
 * grouped into blocks of `block` positions (the last block may be short) and TopK selects
 * BLOCKS, which the following Reuse layers inherit.  The paper does not say how a block is
 * scored from its tokens; the reading taken here is the MAXIMUM over the block's tokens of
 * the group-mean token score (a block matters if it holds a critical token).  Ties go to the
 * lower block; the kb block numbers come out ascending.  The Full layer's output stays the
 * dense attention over all N rows.
 *   bidx   [B, Hkv, kb] int32        bscore (optional) [B, Hkv, ceil(N / block)] double
 */
int hylra_oracle_full_attn_topk_blocks(int kind, int B, int Hq, int Hkv, int d, long N, int block,
                                       int kb, double scale, const void *q, const void *K,
                                       const void *V, double *out, int32_t *bidx, double *bscore)
{
    if (!shape_ok(B, Hq, Hkv, d, N) || block < 1 || !bidx) return ORACLE_BAD_ARG;
    const long nblk = (N + block - 1) / block;
    if (kb < 1 || kb > nblk) return ORACLE_BAD_ARG;
    double *shat = malloc((size_t)B * Hkv * N * sizeof *shat);
    if (!shat) return ORACLE_NOMEM;
    int rc = hylra_oracle_full_attn_topk(kind, B, Hq, Hkv, d, N, 1, scale, q, K, V, out, NULL, shat);
    if (rc != ORACLE_OK) { free(shat); return rc; }
    ranked *r = malloc((size_t)nblk * sizeof *r);
    if (!r) { free(shat); return ORACLE_NOMEM; }
    for (int p = 0; p < B * Hkv; ++p) {
        const double *s = shat + (size_t)p * N;
        for (long c = 0; c < nblk; ++c) {
            const long lo = c * block, hi = lo + block < N ? lo + block : N;
            double m = s[lo];
            for (long j = lo + 1; j < hi; ++j) if (s[j] > m) m = s[j];
            r[c].score = m;
            r[c].pos = (int32_t)c;
            if (bscore) bscore[(size_t)p * nblk + c] = m;
        }
        qsort(r, (size_t)nblk, sizeof *r, by_score_then_pos);
        int32_t *dst = bidx + (size_t)p * kb;
        for (int t = 0; t < kb; ++t) dst[t] = r[t].pos;
        qsort(dst, (size_t)kb, sizeof *dst, by_pos);
    }
    free(r);
    free(shat);
    return ORACLE_OK;
}

/*
 * Reuse layer on inherited BLOCK numbers: attention restricted to every existing token of
 * the named blocks.  Negative block numbers are padding; numbers >= ceil(N / block) are an
 * error.
 */
int hylra_oracle_reuse_block_attn(int kind, int B, int Hq, int Hkv, int d, long N, int block, int kb,
                                  double scale, const void *q, const void *K, const void *V,
                                  const int32_t *bidx, double *out)
{
    if (!shape_ok(B, Hq, Hkv, d, N) || block < 1 || kb < 1 || !bidx || !out) return ORACLE_BAD_ARG;
    const long nblk = (N + block - 1) / block;
    const size_t per = (size_t)kb * block;
    int32_t *tok = malloc((size_t)B * Hkv * per * sizeof *tok);
    if (!tok) return ORACLE_NOMEM;
    for (size_t p = 0; p < (size_t)B * Hkv; ++p)
        for (int t = 0; t < kb; ++t) {
            const int32_t c = bidx[p * kb + t];
            if (c >= nblk) { free(tok); return ORACLE_BAD_ARG; }
            for (int j = 0; j < block; ++j) {
                const long pos = (long)c * block + j;
                tok[p * per + (size_t)t * block + j] = (c < 0 || pos >= N) ? -1 : (int32_t)pos;
            }
        }
    int rc = hylra_oracle_reuse_sparse_attn(kind, B, Hq, Hkv, d, N, (int)per, scale, q, K, V, tok, out);
    free(tok);
    return rc;
}

/* |S_i ∩ S_j| / k for two index sets of size k (overlap ratio, Eq. 2) */
double hylra_oracle_overlap(const int32_t *a, const int32_t *b, int k)
{
    int common = 0;
    for (int i = 0; i < k; ++i)
        for (int j = 0; j < k; ++j)
            if (a[i] >= 0 && a[i] == b[j]) { ++common; break; }
    return (double)common / (double)k;
}

/*
 * Similarity matrix of the offline profiling step (paper: "Inter-Layer Similarity", Eq. 2, and
 * "Similarity Matrix Construction"): for layers i <= j, counts[i * L + j] = the sum over all
 * (batch, KV head) sets of |S_i ∩ S_j|, where S_l is the index set idx_l[l] [B, H, k] of layer
 * l (negative entries are padding).  counts[j * L + i] is left untouched for i < j.
 * Reading (the paper states Eq. 2 for one set per layer): the sets of all sequences and KV
 * heads are pooled, and M[i][j] = counts[i][j] / counts[j][j], so that the diagonal is 1 as
 * the paper sets it.  Plain nested loops.
 */
void hylra_oracle_overlap_counts(int L, int B, int H, int k, const int32_t *const *idx_l, int64_t *counts)
{
    for (int i = 0; i < L; ++i)
        for (int j = i; j < L; ++j) {
            int64_t total = 0;
            for (int s = 0; s < B * H; ++s) {
                const int32_t *a = idx_l[i] + (size_t)s * k, *b = idx_l[j] + (size_t)s * k;
                for (int x = 0; x < k; ++x) {
                    if (a[x] < 0) continue;
                    for (int y = 0; y < k; ++y)
                        if (a[x] == b[y]) { ++total; break; }
                }
            }
            counts[(size_t)i * L + j] = total;
        }
}

/*
 * Offline policy search (paper: Algorithm 1 "Offline Policy Optimization via Dynamic
 * Programming" and the section of that name).  M [L][L] row-major, M[i][j] for source layer
 * i <= target layer j; theta the similarity threshold.
 *
 * A state (i, j), i <= j, means layer j uses the index set of layer i (i == j: full
 * attention at j).  Every state keeps its best path value (C, S): C = number of
 * full-attention layers on the path, S = sum of M over the path's states; better means
 * smaller C, then larger S.  The path starts at (0, 0) with C = 1, S = M[0][0] (layer 0
 * computes full attention; reading: it counts).  From (i, j): the vertical move to (i, j+1)
 * is allowed if M[i][j+1] >= theta and adds M[i][j+1] to S; the reset jump to (j+1, j+1)
 * adds 1 to C and M[j+1][j+1] to S.  A candidate replaces the state's value only if it is
 * strictly better, and candidates arrive in the order of the algorithm's loops (j ascending,
 * i ascending, vertical move before reset jump), so among equal values the first one stays
 * (the paper does not say; reading).  The answer is the best state of the last layer (first
 * one among equals), traced back: policy[l] = 0 (Full) for diagonal states, 1 (Reuse) else.
 * Returns the number of Full layers C*, and S* through sum_sim.
 */
int hylra_oracle_policy_search(int L, const double *M, double theta, uint8_t *policy, double *sum_sim)
{
    /* value and predecessor (source index at layer j-1) of state (i, j) */
    int *C = malloc(sizeof(int) * L * L), *prev = malloc(sizeof(int) * L * L);
    double *S = malloc(sizeof(double) * L * L);
    char *reach = calloc((size_t)L * L, 1);
    C[0] = 1, S[0] = M[0], prev[0] = -1, reach[0] = 1;
    for (int j = 0; j + 1 < L; ++j)
        for (int i = 0; i <= j; ++i) {
            if (!reach[i * L + j]) continue;
            const int c = C[i * L + j];
            const double s = S[i * L + j];
            /* vertical move: index reuse */
            if (M[i * L + j + 1] >= theta) {
                const int t = i * L + j + 1;
                const double cs = s + M[i * L + j + 1];
                if (!reach[t] || c < C[t] || (c == C[t] && cs > S[t])) {
                    reach[t] = 1, C[t] = c, S[t] = cs, prev[t] = i;
                }
            }
            /* reset jump: full attention */
            {
                const int t = (j + 1) * L + j + 1;
                const double cs = s + M[t];
                if (!reach[t] || c + 1 < C[t] || (c + 1 == C[t] && cs > S[t])) {
                    reach[t] = 1, C[t] = c + 1, S[t] = cs, prev[t] = i;
                }
            }
        }
    int best = -1;
    for (int i = 0; i < L; ++i) {
        const int t = i * L + L - 1;
        if (!reach[t]) continue;
        if (best < 0 || C[t] < C[best * L + L - 1] || (C[t] == C[best * L + L - 1] && S[t] > S[best * L + L - 1]))
            best = i;
    }
    const int c_star = best >= 0 ? C[best * L + L - 1] : 0;   /* (the last layer is always reachable by reset jumps) */
    if (sum_sim) *sum_sim = S[best * L + L - 1];
    for (int j = L - 1, i = best; j >= 0; --j) {
        policy[j] = (i == j) ? 0 : 1;
        i = prev[i * L + j];
    }
    free(C), free(prev), free(S), free(reach);
    return c_star;
}

int hylra_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
