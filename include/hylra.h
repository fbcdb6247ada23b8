/*
 * libhylra -- the per-layer decode-attention step of HyLRA (Hybrid Layer Reuse
 * Attention) for one MI355X (gfx950), as a C ABI.
 *
 * The operations follow the paper's Algorithm 2 ("Hybrid Inter-Layer Top-K Reuse
 * Attention") with attention as in Eq. 1:
 *
 *   Full layer   S = q K^T / sqrt(d);  I = TopK(S, k);  O = Softmax(S) V over ALL rows
 *   Reuse layer  I inherited from the previous layer;  O = Attention(q, K[I], V[I])
 *   Step         the layers in order, a policy vector choosing the branch per layer
 *
 * The paper states the algorithm for one head.  Here several query heads may
 * share one KV head (query head h reads KV head h / G, G = n_q_heads /
 * n_kv_heads) and there is ONE index set per (batch, KV head): positions are
 * ranked by the mean over the group's G heads of the scaled scores; ties go to
 * the lower position; the k positions are written in ascending order.
 *
 * General conventions
 *   - Every tensor pointer is a DEVICE pointer owned by the caller unless marked
 *     HOST.  The library never frees or keeps caller memory.
 *   - q   bf16 [B, Hq, d] contiguous.   K, V  bf16 [B, Hkv, N, d] addressed through
 *     the element strides in hylra_shape (innermost dimension contiguous).
 *     out fp32 [B, Hq, d] contiguous.   idx  int32 [B, Hkv, k] contiguous.
 *   - K, V, q must be 16-byte aligned and the strides multiples of 8 elements.
 *   - All work is enqueued on the given HIP stream (a hipStream_t passed as void*,
 *     NULL = the default stream) and is asynchronous with respect to the host.
 *     No call below allocates, synchronises or copies to the host, except
 *     hylra_create / hylra_destroy and the hylra_profile_* / hylra_probe_* aids.
 *   - A context owns a fixed device workspace sized at creation for a maximum
 *     shape; calls with a larger shape fail with HYLRA_ERR_WORKSPACE.  A context
 *     serves one stream at a time: concurrent calls on one context race on the
 *     workspace.
 *   - Errors are return codes; arguments are checked before anything is launched.
 *     hylra_last_error() gives the detail text of the most recent failure.
 */
#ifndef HYLRA_H
#define HYLRA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hylra_ctx hylra_ctx;

typedef enum {
    HYLRA_OK = 0,
    HYLRA_ERR_BAD_ARG = 1,     /* null pointer, misaligned tensor, k outside 1..N, ...      */
    HYLRA_ERR_UNSUPPORTED = 2, /* head_dim not 64/128, group size above 8, ...               */
    HYLRA_ERR_WORKSPACE = 3,   /* shape or k larger than what the context was created for    */
    HYLRA_ERR_POLICY = 4,      /* policy[0] is not Full, or an entry is neither 0 nor 1      */
    HYLRA_ERR_HIP = 5          /* a HIP runtime call failed (text in hylra_last_error)       */
} hylra_status;

#define HYLRA_FULL 0
#define HYLRA_REUSE 1

typedef struct {
    int32_t batch;       /* B                                                              */
    int32_t n_q_heads;   /* Hq, a multiple of n_kv_heads; Hq / Hkv <= 8                     */
    int32_t n_kv_heads;  /* Hkv                                                            */
    int32_t head_dim;    /* d: 64 or 128                                                   */
    int32_t ctx_len;     /* N: rows in the KV cache (includes the current token)           */
    int64_t kv_stride_b; /* element strides of K and V; all three 0 => contiguous [B,Hkv,N,d] */
    int64_t kv_stride_h;
    int64_t kv_stride_n;
    float scale;         /* score scale; 0 => 1/sqrt(head_dim) (Eq. 1)                     */
} hylra_shape;

/* Creates a context on HIP device `device` with a workspace large enough for
 * any call whose shape is <= max_shape in every extent and whose k <= max_k.
 * HOST call; allocates device memory; *out is NULL on failure. */
hylra_status hylra_create(hylra_ctx **out, const hylra_shape *max_shape, int32_t max_k, int device);

/*
 * hylra_create with behaviour flags (hylra_create passes 0):
 *   HYLRA_FLAG_DETERMINISTIC  only kernels whose every output is bit-identical from run to run.
 *       Without it the Full layer may hand its rows out to workgroups at run time (faster on
 *       large batches); index sets and Reuse outputs are bit-reproducible either way, but the
 *       Full layer's attention output can then differ in the last bits between runs (the
 *       partial sums are formed in a different grouping), within 1e-5 relative.
 *   HYLRA_FLAG_TOPK_EVERY_FULL_LAYER  hylra_decode_step* run TopK at every Full layer, as
 *       Algorithm 2 is written, also where the set would be overwritten before anyone reads
 *       it (a Full layer directly followed by another).  Outputs are the same either way.
 */
#define HYLRA_FLAG_DETERMINISTIC 1u
#define HYLRA_FLAG_TOPK_EVERY_FULL_LAYER 2u
hylra_status hylra_create_ex(hylra_ctx **out, const hylra_shape *max_shape, int32_t max_k, int device,
                             uint32_t flags);

/* Frees the workspace.  The caller makes sure no work of this context is still
 * running.  NULL is accepted. */
hylra_status hylra_destroy(hylra_ctx *ctx);

/* Puts the context's workspace back into its initial state: synchronises the device, zeroes the
 * counters and histograms the kernels keep between launches, clears the sticky error below.
 * HOST call.  Needed only after a call failed with the text "gave up waiting": the Full
 * kernels that hand rows out at run time, the one-launch top-k selection and the Reuse kernels
 * that merge by packets bound every wait; should such a wait ever run out (it cannot unless the device is failing or
 * two calls on one context overlapped), the launch's results are incomplete, the context
 * records it, and every later call on the context fails with HYLRA_ERR_HIP until hylra_reset. */
hylra_status hylra_reset(hylra_ctx *ctx);

/* Static, never NULL. */
const char *hylra_status_str(hylra_status s);

/* Detail text of the last failing call on this context (owned by the context,
 * valid until the next call).  "" if none.  With ctx == NULL: the text of the
 * last failed hylra_create on this thread. */
const char *hylra_last_error(const hylra_ctx *ctx);

/*
 * Full layer (Algorithm 2, Full branch; Eq. 1).
 *   out[b,h,:]  = sum_j softmax_j(scale * q[b,h,:].K[b,h/G,j,:]) * V[b,h/G,j,:]   over all N rows
 *   idx[b,g,:]  = the k positions j with the largest mean_h-in-group(scale * q.K_j),
 *                 ties to the lower position, ascending order
 * One streaming pass over K and V; scores are computed in fp32 from the bf16
 * inputs (products exact, fp32 accumulation).  Requires 1 <= k <= N.
 */
hylra_status hylra_full_attn_topk(hylra_ctx *ctx, const hylra_shape *shape,
                                  const void *q, const void *K, const void *V, int32_t k,
                                  float *out, int32_t *idx, void *hip_stream);

/*
 * Reuse layer (Algorithm 2, Reuse branch): attention restricted to the rows
 * named by idx[b, g, 0..k-1], shared by the G query heads of KV head g.
 * Entries that are negative or >= N are skipped (padding); a set with no valid
 * entry gives a zero output row.  Only the selected rows of K and V are read.
 */
hylra_status hylra_reuse_sparse_attn(hylra_ctx *ctx, const hylra_shape *shape,
                                     const void *q, const void *K, const void *V,
                                     const int32_t *idx, int32_t k, float *out,
                                     void *hip_stream);

/*
 * hylra_reuse_sparse_attn for callers that cannot allocate device memory at all (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): no context, and
 * no allocation inside -- neither hipMalloc / hipFree nor any allocating library routine.
 * The split partials and arrival counters that the other entry points keep in a context's
 * workspace live in a fixed array inside the library's device image instead (about 2.1 MB,
 * held by every GPU the library has been loaded on until the process ends).  Runs on the
 * CURRENT HIP device; hip_stream must belong to it.  Arguments, results and numerics are those
 * of hylra_reuse_sparse_attn (same kernels, same split plan).
 * Limits: batch * n_kv_heads <= 2048 and batch * n_q_heads * splits <= 4096, where splits is
 * the number of workgroups the plan gives one (batch, KV head) (every benchmark shape fits);
 * anything larger fails with HYLRA_ERR_WORKSPACE before a kernel is launched.  Failures leave
 * their text in hylra_last_error(NULL) (per thread).
 * All calls on one GPU share the one array: calls that overlap in time on one GPU (two
 * streams, two threads) race on it; calls on one stream, or otherwise ordered, do not.  The
 * array keeps the previous call's contents; the call clears what it needs cleared.
 */
hylra_status hylra_reuse_sparse_attn_static(const hylra_shape *shape, const void *q, const void *K,
                                            const void *V, const int32_t *idx, int32_t k,
                                            float *out, void *hip_stream);

/*
 * One decode step over n_layers layers (Algorithm 2, outer loop), in order, on
 * one stream.  policy is a HOST array: HYLRA_FULL runs hylra_full_attn_topk and
 * overwrites idx_buf; HYLRA_REUSE runs hylra_reuse_sparse_attn on idx_buf as the
 * most recent Full layer left it.  policy[0] must be HYLRA_FULL.
 * q_l, K_l, V_l, out_l are HOST arrays of n_layers DEVICE pointers (read during
 * the call only).  idx_buf is DEVICE memory of at least B*Hkv*k int32; on return
 * (stream order) it holds the last Full layer's set.  A Full layer directly
 * followed by another Full layer hands its set to no one; its TopK is skipped
 * (its output is computed as always).
 */
hylra_status hylra_decode_step(hylra_ctx *ctx, const hylra_shape *shape, int32_t n_layers,
                               const uint8_t *policy, const void *const *q_l,
                               const void *const *K_l, const void *const *V_l, int32_t k,
                               float *const *out_l, int32_t *idx_buf, void *hip_stream);

/*
 * Block-level variant (paper, section on hardware-efficient optimizations, adaptation to
 * block-level sparsity): consecutive rows of the cache form blocks of `block` rows (the last
 * block may be short) and TopK ranks BLOCKS; Reuse layers inherit the block numbers and
 * attend to every row of the named blocks.  The paper does not fix how a block is scored
 * from its rows; here a block scores the MAXIMUM of its rows' group-mean scaled logits.
 * Ties go to the lower block; numbers come out ascending.  The Full layer's output is the
 * dense attention over all ctx_len rows, as in hylra_full_attn_topk.
 *
 *   block   rows per block, 1..65536 (1 = the token-level calls above); any value, not only
 *           powers of two
 *   kb      blocks selected per (batch, KV head): 1..ceil(ctx_len / block), and
 *           kb * block <= max_k of hylra_create rounded up to a multiple of block
 *   bidx    DEVICE [batch, n_kv_heads, kb] int32: written by the Full call, read by the
 *           Reuse call.  For the Reuse call, entries < 0 or >= ceil(ctx_len / block) are
 *           padding and skipped, as are the rows of the last block beyond ctx_len.
 *   bidx_buf  DEVICE, at least batch * n_kv_heads * kb int32 (as idx_buf above)
 * All other arguments, ownership, stream order and error behaviour are those of the
 * token-level calls of the same name.
 */
hylra_status hylra_full_attn_topk_blocks(hylra_ctx *ctx, const hylra_shape *shape, const void *q,
                                         const void *K, const void *V, int32_t block, int32_t kb,
                                         float *out, int32_t *bidx, void *hip_stream);
hylra_status hylra_reuse_block_attn(hylra_ctx *ctx, const hylra_shape *shape, const void *q,
                                    const void *K, const void *V, const int32_t *bidx,
                                    int32_t block, int32_t kb, float *out, void *hip_stream);
hylra_status hylra_decode_step_blocks(hylra_ctx *ctx, const hylra_shape *shape, int32_t n_layers,
                                      const uint8_t *policy, const void *const *q_l,
                                      const void *const *K_l, const void *const *V_l, int32_t block,
                                      int32_t kb, float *const *out_l, int32_t *bidx_buf,
                                      void *hip_stream);

/*
 * Paged KV cache and per-sequence lengths: the same three operations for the cache
 * layout of a serving engine (the method keeps the full KV cache and only changes
 * what is read from it; it says nothing about the cache's layout or about batches
 * of sequences of different lengths, so the reading is: sequence b attends to and
 * ranks its own first n_b rows).
 *
 * K_pool, V_pool: bf16 pools of pages; page p, KV head g, token slot s starts at
 * element  p * stride_page + g * stride_head + s * stride_row  (innermost
 * dimension contiguous; strides multiples of 8 elements, stride_row >= head_dim).
 * block_table[b][t] (DEVICE, int32, max_pages columns) names the page holding rows
 * t * page_size .. (t + 1) * page_size - 1 of sequence b; only the entries that
 * cover rows 0 .. n_b - 1 are read, and those must name pages inside the pools
 * (the library cannot check device-resident page numbers before it launches).
 * seq_lens[b] (DEVICE, int32) is n_b, clamped
 * to 0 .. shape->ctx_len; NULL means n_b = shape->ctx_len for every sequence.
 * shape->ctx_len is the largest length a sequence of the call may have (it sizes
 * the launch); shape's kv strides are ignored.  One table serves K and V, and in
 * hylra_decode_step_paged every layer (each layer has its own pools).
 * block_table == NULL means a contiguous cache with per-sequence lengths only:
 * K_pool / V_pool are then K and V addressed through shape's strides, as in the
 * calls above, and page_size, max_pages and the pool strides are ignored.
 *
 * Full layer: sequence b selects min(k, n_b) rows; idx[b, g, min(k, n_b) .. k-1]
 * = -1.  A sequence with n_b = 0 gets a zero output row and no index.  Requires
 * 1 <= k <= shape->ctx_len.  Reuse layer: entries < 0 or >= n_b are padding.
 */
typedef struct {
    int32_t page_size;          /* rows per page: a power of two, 1 .. 65536                */
    int32_t max_pages;          /* columns of block_table; >= ceil(ctx_len / page_size)     */
    int64_t stride_page;        /* element strides of the pools, see above                  */
    int64_t stride_head;
    int64_t stride_row;
    const int32_t *block_table; /* DEVICE [batch][max_pages]; NULL: contiguous cache           */
    const int32_t *seq_lens;    /* DEVICE [batch], or NULL                                  */
} hylra_paged;

hylra_status hylra_full_attn_topk_paged(hylra_ctx *ctx, const hylra_shape *shape,
                                        const hylra_paged *cache, const void *q,
                                        const void *K_pool, const void *V_pool, int32_t k,
                                        float *out, int32_t *idx, void *hip_stream);

hylra_status hylra_reuse_sparse_attn_paged(hylra_ctx *ctx, const hylra_shape *shape,
                                           const hylra_paged *cache, const void *q,
                                           const void *K_pool, const void *V_pool,
                                           const int32_t *idx, int32_t k, float *out,
                                           void *hip_stream);

/* As hylra_decode_step, with K_pool_l[l] / V_pool_l[l] the pools of layer l. */
hylra_status hylra_decode_step_paged(hylra_ctx *ctx, const hylra_shape *shape,
                                     const hylra_paged *cache, int32_t n_layers,
                                     const uint8_t *policy, const void *const *q_l,
                                     const void *const *K_pool_l, const void *const *V_pool_l,
                                     int32_t k, float *const *out_l, int32_t *idx_buf,
                                     void *hip_stream);

/*
 * The block-level variant on a paged cache or with per-sequence lengths: blocks are
 * `block` consecutive rows of a sequence (they need not line up with pages); sequence b
 * has ceil(n_b / block) of them, the last one possibly short, selects
 * min(kb, ceil(n_b / block)) and pads its index entries with -1.  Arguments as in the
 * calls of the same names above.
 */
hylra_status hylra_full_attn_topk_blocks_paged(hylra_ctx *ctx, const hylra_shape *shape,
                                               const hylra_paged *cache, const void *q,
                                               const void *K_pool, const void *V_pool, int32_t block,
                                               int32_t kb, float *out, int32_t *bidx, void *hip_stream);
hylra_status hylra_reuse_block_attn_paged(hylra_ctx *ctx, const hylra_shape *shape,
                                          const hylra_paged *cache, const void *q,
                                          const void *K_pool, const void *V_pool, const int32_t *bidx,
                                          int32_t block, int32_t kb, float *out, void *hip_stream);
hylra_status hylra_decode_step_blocks_paged(hylra_ctx *ctx, const hylra_shape *shape,
                                            const hylra_paged *cache, int32_t n_layers,
                                            const uint8_t *policy, const void *const *q_l,
                                            const void *const *K_pool_l, const void *const *V_pool_l,
                                            int32_t block, int32_t kb, float *const *out_l,
                                            int32_t *bidx_buf, void *hip_stream);

/*
 * Index-guided prefetch ("Bandwidth reduction via index-guided offloading"): when
 * a tolerant layer's cache lives in memory the GPU reads slowly (pinned host memory
 * across PCIe), its index set is known as soon as the preceding Full layer has
 * run, so only the selected rows are fetched, ahead of time.
 *
 * hylra_gather_rows: K_src / V_src are addressed as K and V of shape (any memory
 * the device can read); idx DEVICE int32 [B, Hkv, k].  Writes, in DEVICE memory,
 *   K_dst[b,g,t,:] = K_src[b,g,idx[b,g,t],:]   (bf16 [B,Hkv,k,d] contiguous; likewise V_dst;
 *                                               zero rows where idx holds padding)
 *   idx_dst[b,g,t] = t, or -1 where idx[b,g,t] is < 0 or >= ctx_len
 * so that hylra_reuse_sparse_attn over (K_dst, V_dst, idx_dst) with ctx_len = k
 * equals hylra_reuse_sparse_attn over (K_src, V_src, idx).
 *
 * hylra_decode_step_offloaded: hylra_decode_step with the Reuse layers' K_l[l] /
 * V_l[l] in such slow memory (Full layers' caches in device memory).  Gathers run
 * on copy_stream into slots of a DEVICE staging buffer and overlap the attention
 * kernels on compute_stream; the two are ordered by events the context owns.
 * staging holds staging_bytes / hylra_offload_slot_bytes(shape, k) >= 1 slots; with
 * s slots up to s layers are prefetched ahead.  The streams may be the same (no
 * overlap then).  On return both streams have the work enqueued; results are
 * complete when compute_stream has drained.  n_layers <= 256.
 *
 * Block granularity and paged caches (the paper prefetches "only the critical KV blocks"):
 * hylra_gather_blocks and hylra_decode_step_offloaded_blocks are the two calls above for the
 * block-level variant (block rows per block, kb blocks per (batch, KV head); block = 1 is the
 * token level) and for any cache layout (cache as in the *_paged calls: paged pools and / or
 * per-sequence lengths; NULL = contiguous through shape's strides).  Slot t * block + r of the
 * compact cache receives row bidx[b,g,t] * block + r of sequence b, or zeros and index entry -1
 * where that is no row of the sequence (padding entry, block number out of range, row at or
 * past the sequence's length); K_dst / V_dst are [B, Hkv, kb * block, d], idx_dst
 * [B, Hkv, kb * block].  In the step, whole blocks (block * head_dim * 2 bytes of K and of V,
 * contiguous in the source unless a block straddles pages) cross the slow link; the block
 * table and the lengths are DEVICE arrays as always, only the Reuse layers' pools are in slow
 * memory.  A slot holds hylra_offload_slot_bytes(shape, kb * block) bytes; kb * block <= max_k.
 */
size_t hylra_offload_slot_bytes(const hylra_shape *shape, int32_t k);
hylra_status hylra_gather_rows(hylra_ctx *ctx, const hylra_shape *shape, const void *K_src,
                               const void *V_src, const int32_t *idx, int32_t k, void *K_dst,
                               void *V_dst, int32_t *idx_dst, void *hip_stream);
hylra_status hylra_decode_step_offloaded(hylra_ctx *ctx, const hylra_shape *shape, int32_t n_layers,
                                         const uint8_t *policy, const void *const *q_l,
                                         const void *const *K_l, const void *const *V_l, int32_t k,
                                         float *const *out_l, int32_t *idx_buf, void *staging,
                                         size_t staging_bytes, void *compute_stream,
                                         void *copy_stream);

hylra_status hylra_gather_blocks(hylra_ctx *ctx, const hylra_shape *shape, const hylra_paged *cache,
                                 const void *K_src, const void *V_src, const int32_t *bidx,
                                 int32_t block, int32_t kb, void *K_dst, void *V_dst,
                                 int32_t *idx_dst, void *hip_stream);
hylra_status hylra_decode_step_offloaded_blocks(hylra_ctx *ctx, const hylra_shape *shape,
                                                const hylra_paged *cache, int32_t n_layers,
                                                const uint8_t *policy, const void *const *q_l,
                                                const void *const *K_l, const void *const *V_l,
                                                int32_t block, int32_t kb, float *const *out_l,
                                                int32_t *bidx_buf, void *staging, size_t staging_bytes,
                                                void *compute_stream, void *copy_stream);

/*
 * Append, then attend: Algorithm 2 takes K^cache and V^cache with the current token already
 * in them.  These calls first write the token's key and value, k_new / v_new (DEVICE, bf16
 * [B, Hkv, d] contiguous, 16-byte aligned), into the cache and then run the attention of the
 * same name over the cache including that row, as one launch sequence on the stream.
 *   cache == NULL, or cache->seq_lens == NULL: every sequence has ctx_len - 1 rows before the
 *     call; the token becomes row ctx_len - 1 and the attention covers ctx_len rows.
 *   cache->seq_lens given: seq_lens[b] = n_b is the length BEFORE the call (clamped to
 *     0 .. ctx_len - 1); the token becomes row n_b of sequence b -- through block_table[b] if
 *     the cache is paged, whose page for that row the caller has allocated -- and sequence b
 *     attends to and ranks n_b + 1 rows.  seq_lens itself is not written; the caller advances
 *     its lengths after the step.
 * K, V (pools if paged) are written: one row of each per (batch, KV head).  Everything else --
 * arguments, selection rule, padding of short sequences, errors -- is as in
 * hylra_full_attn_topk_paged / hylra_reuse_sparse_attn_paged / hylra_decode_step_paged.  In
 * hylra_decode_step_append every layer l gets its own k_new_l[l], v_new_l[l] (HOST arrays of
 * DEVICE pointers) written into its own cache before the layer's attention.  A Reuse layer
 * attends to the inherited set as it is (the new row takes part if the set names it).
 * Launches: the Reuse form is ONE launch -- the matrix-core Reuse kernels read the new row from
 * k_new / v_new wherever the set names it and write it into the cache themselves (option
 * "append_unfused" = 1, and the vector Reuse kernel always: a small launch writes the rows
 * first); the Full form is that small launch followed by the Full layer's own launches.
 */
hylra_status hylra_append_full_attn_topk(hylra_ctx *ctx, const hylra_shape *shape,
                                         const hylra_paged *cache, const void *q,
                                         const void *k_new, const void *v_new, void *K, void *V,
                                         int32_t k, float *out, int32_t *idx, void *hip_stream);
hylra_status hylra_append_reuse_sparse_attn(hylra_ctx *ctx, const hylra_shape *shape,
                                            const hylra_paged *cache, const void *q,
                                            const void *k_new, const void *v_new, void *K, void *V,
                                            const int32_t *idx, int32_t k, float *out,
                                            void *hip_stream);
hylra_status hylra_decode_step_append(hylra_ctx *ctx, const hylra_shape *shape,
                                      const hylra_paged *cache, int32_t n_layers,
                                      const uint8_t *policy, const void *const *q_l,
                                      const void *const *k_new_l, const void *const *v_new_l,
                                      void *const *K_l, void *const *V_l, int32_t k,
                                      float *const *out_l, int32_t *idx_buf, void *hip_stream);

/*
 * Offline profiling: from the index sets of an all-Full run to the layer policy
 * ("Inter-Layer Similarity", Eq. 2; "Offline Optimal Policy via Dynamic
 * Programming", Algorithm 1).
 *
 * hylra_overlap_counts: idx_l is a HOST array of n_layers (<= 256) DEVICE
 * pointers, idx_l[l] = the int32 [batch, n_kv_heads, k] index set layer l's Full
 * attention produced (entries < 0 or >= ctx_len are padding; ctx_len <= 524288).
 * counts (DEVICE, int64 [n_layers][n_layers]) receives, for i <= j,
 * counts[i][j] = the sum over all (batch, KV head) sets of |S_i ∩ S_j|; entries
 * below the diagonal are set to zero.  Enqueued on the stream.
 *
 * hylra_similarity_matrix (HOST arrays): M[i][j] = counts[i][j] / counts[j][j] for
 * i <= j (the diagonal is 1, as the paper sets it; a layer without valid entries
 * gets 0 off the diagonal), 0 below the diagonal.
 *
 * hylra_policy_search (HOST arrays, no GPU work, ctx may be NULL): the path
 * search of Algorithm 1 over M [n_layers][n_layers] (source layer i <= target
 * layer j) with threshold theta: fewest Full layers first, then the largest sum of
 * similarities along the path; layer 0 is Full and counts; among equal values the
 * candidate met first in the order of the algorithm's loops is kept.  policy[l]
 * receives HYLRA_FULL or HYLRA_REUSE; n_full and sum_sim (either may be NULL) the
 * value of the chosen path.
 */
hylra_status hylra_overlap_counts(hylra_ctx *ctx, int32_t n_layers, const int32_t *const *idx_l,
                                  int32_t batch, int32_t n_kv_heads, int32_t k, int32_t ctx_len,
                                  int64_t *counts, void *hip_stream);
hylra_status hylra_similarity_matrix(int32_t n_layers, const int64_t *counts, double *M);
hylra_status hylra_policy_search(hylra_ctx *ctx, int32_t n_layers, const double *M, double theta,
                                 uint8_t *policy, int32_t *n_full, double *sum_sim);

/*
 * Tuning knobs (HOST call, takes effect for later launches).  Unknown names give
 * HYLRA_ERR_BAD_ARG; 0 always means "automatic / default".  Names:
 *   "full_split_rows"   rows of the cache per workgroup of the Full kernel (the vector-ALU
 *                       kernels take at most 8192 and clamp larger values)
 *   "reuse_split_rows"  index entries per workgroup of the Reuse kernel
 *   "full_variant"      Full streaming kernel.  Vector-ALU kernel (two-deep register pipeline,
 *                       streaming loads): 23 = even splits, 43 = rows handed out at run time.
 *                       First matrix-core kernel: 52.  Second matrix-core kernel (head_dim 128):
 *                       72 = even splits, 74 = rows handed out at run time.  Defaults: head_dim
 *                       128: 74 while batch * n_kv_heads >= 64 (up to 4 heads per KV head) or
 *                       whenever the launch has exactly two workgroups per compute unit, 72
 *                       otherwise and for small problems (under 2048 rows per workgroup);
 *                       head_dim 64: 52 from 5 heads per KV head, else 43 while batch *
 *                       n_kv_heads >= 64 and 23 below that.  HYLRA_FLAG_DETERMINISTIC rules out
 *                       43 and 74 as defaults (see hylra_create_ex).
 *   "reuse_variant"     Reuse gather kernel: 1 / 2 = vector-ALU kernel with streaming / plain
 *                       loads, 3 / 4 = first matrix-core kernel with streaming / plain loads
 *                       (default for head_dim 64: 4), 5 / 6 = second matrix-core kernel
 *                       (head_dim 128 only; default there: 5)
 *   "reuse_unroll"      row groups per wave tile of the Reuse kernel: 1, 2, 4 or 8 (the second
 *                       matrix-core kernel: 4 = wave tiles of 32 rows, otherwise of 64)
 *   "reuse_waves"       waves per workgroup of the matrix-core Reuse kernel: 4 or 8
 *   "reuse_merge"       how the Reuse kernel merges the partials of a (batch, KV head) across
 *                       workgroups.  0 = automatic; 1 = always by arrival counter (the last
 *                       workgroup to arrive merges everything); 2 = by packets (every workgroup
 *                       merges a slice of the columns) whenever the launch allows it: head_dim
 *                       128, 4 .. 128 partials per pair and a power of two, no more workgroups
 *                       than compute units.  Automatic: packets from 8 partials on, and with
 *                       few (batch, KV head) pairs twice as many workgroups with wave tiles of
 *                       32 rows.  The workgroups of such a launch wait for one another (bounded:
 *                       see hylra_reset), which needs all of them resident at once: a launch
 *                       puts at most one workgroup of 4 or 8 waves on a compute unit (which holds
 *                       32), so several can share the device, but a device kept full by other
 *                       long-running work is a reason to set 1.
 *   "reuse_unfused"     1 = merge the Reuse partials in a second kernel instead of in the
 *                       last-arriving workgroup of the Reuse kernel
 *   "simulate_give_up"  1 = mark the context as if a kernel had given up a bounded wait (for
 *                       tests of that error path; see hylra_reset)
 *   "append_unfused"    1 = hylra_append_reuse_sparse_attn and the Reuse layers of
 *                       hylra_decode_step_append write the new rows with a launch of their own
 *                       instead of inside the Reuse kernel
 *   "topk_two_launches" 1 = the top-k selection after the streaming pass always runs as two
 *                       launches (scan, emit).  Default: one launch when it has no more
 *                       workgroups than the device has compute units (its workgroups wait for one
 *                       another's counts, bounded: see hylra_reset), two otherwise.
 *   "hist_unfused"      1 = the first histogram of the top-k selection is made by a launch of
 *                       its own instead of inside the Full layer's streaming kernel
 *   "full_unpaired"     1 = the self-scheduling Full kernels group their workgroups by number
 *                       instead of mixing early and late arrivals on the compute units
 *   "ragged_even"       1 = with seq_lens, give every (batch, KV head) the same number of
 *                       workgroups of the self-scheduling Full kernel instead of a number in
 *                       proportion to its rows
 */
hylra_status hylra_set_option(hylra_ctx *ctx, const char *name, int32_t value);

/*
 * What the library decided for the most recent launches of the context, for tests and for
 * tuning.  *value (HOST) receives, for the most recent Reuse-layer launch ("Sparse Attention",
 * Algorithm 2's Reuse branch):
 *   "last_reuse_splits"     workgroups (= partials) per (batch, KV head)
 *   "last_reuse_wave_rows"  index entries a wave takes per sweep (matrix-core kernels: 32 or 64)
 *   "last_reuse_merge"      how the partials met: 0 = a second kernel, 1 = arrival counter,
 *                           2 = packets, 3 = one workgroup per pair, nothing to merge
 * and for the most recent Full-layer call ("TopK", Algorithm 2's Full branch):
 *   "last_topk_launches"    launches of the selection after the streaming pass: 1, 2, or 0 if
 *                           the layer's index set was not wanted
 * 0 everywhere before the first such launch.  An unknown name is HYLRA_ERR_BAD_ARG.
 */
hylra_status hylra_get_info(const hylra_ctx *ctx, const char *name, int32_t *value);

/*
 * Measurement aids (not on the hot path).
 *
 * hylra_profile_enable(ctx, 1) makes every later kernel launch of this context
 * be bracketed by a pair of HIP events on the launch stream (consecutive
 * launches of one class on one stream share one pair, so a launch is charged
 * what it costs back to back); hylra_profile_read synchronises those events
 * and returns, per kernel class, the number of launches and the summed
 * duration in milliseconds since the last hylra_profile_reset.  Classes: 0 = Full attention (split-KV pass),
 * 1 = Full finalise (combine + top-k; all its launches), 2 = Reuse attention, 3 = Reuse combine (absent
 * in the fused mode), 4 = probe kernels.  At most HYLRA_PROFILE_MAX_EVENTS event pairs are recorded
 * between resets; later launches run untimed.
 */
#define HYLRA_PROFILE_CLASSES 5
#define HYLRA_PROFILE_MAX_EVENTS 4096
hylra_status hylra_profile_enable(hylra_ctx *ctx, int32_t on);
hylra_status hylra_profile_reset(hylra_ctx *ctx);
hylra_status hylra_profile_read(hylra_ctx *ctx, int32_t kernel_class, int32_t *n_launches,
                                double *total_ms);

/* Plain device-to-device copy kernel of `bytes` bytes (a multiple of 16; both
 * pointers 16-byte aligned): the known-size reference against which hardware
 * traffic counters are scaled. */
hylra_status hylra_probe_copy(hylra_ctx *ctx, void *dst, const void *src, size_t bytes,
                              void *hip_stream);

/* Streaming read of `bytes` bytes (multiple of 16; non-temporal loads, as the attention
 * kernels read the cache) with a trivial reduction;
 * writes one 32-bit word per workgroup to `sink` (>= 16384 bytes).  Measures the
 * reachable HBM read rate. */
hylra_status hylra_probe_read(hylra_ctx *ctx, const void *src, size_t bytes, void *sink,
                              void *hip_stream);

/* Bare gather of the rows a Reuse layer over (K, V, idx, k) would read -- the same bytes,
 * fetched whole rows at a time with everything in flight at once, and no arithmetic: the
 * floor under hylra_reuse_sparse_attn for these index sets.  Arguments as in
 * hylra_reuse_sparse_attn; entries < 0 or >= ctx_len are skipped; sink (>= 16384 bytes,
 * 16-byte aligned) is practically never written. */
hylra_status hylra_probe_gather(hylra_ctx *ctx, const hylra_shape *shape, const void *K,
                                const void *V, const int32_t *idx, int32_t k, void *sink,
                                void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* HYLRA_H */
