// Internal interface between the host API and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "host_logic.h"

namespace hylra {

constexpr int kMaxGroup = 8;        // query heads per KV head
constexpr int kMaxSplits = 1024;    // partials per (batch, KV head) the finalise kernels accept
constexpr int kMaxFullSplitRows = 8192;   // rows per workgroup of the vector Full kernel (its scores sit in LDS)
constexpr int kCtrStride = 64;      // ints between the chunk counters of two (batch, KV head) pairs

// Where the rows of the cache live and how many a sequence has (paged caches and
// per-sequence lengths; a serving engine keeps the cache in fixed-size pages and batches
// sequences of different lengths).  table == nullptr: sequence b is the contiguous range of
// rows starting at b * sb.  Otherwise rows t * 2^page_shift .. of sequence b are the rows of
// page table[b * table_stride + t], and sb is unused.
struct RowMap {
    const int32_t* table;
    const int32_t* seq_lens;        // [B] rows of sequence b, clamped to 0..N; nullptr: N everywhere
    int table_stride, page_shift;
    int64_t stride_page;            // elements between two pages of a pool
};

struct FullParams {
    const uint16_t* q;
    const uint16_t* K;
    const uint16_t* V;
    int64_t sb, sh, sn;             // element strides of K and V (sn: between rows, also inside a page)
    RowMap map;
    int tbl_cap;                    // page-table entries a workgroup can stage in LDS (0 if not paged)
    int Hq, Hkv, N;
    int rows_per_split, n_splits;
    float scale_log2;               // scale * log2(e)
    float scale_mean;               // scale / G
    float* part_ml;                 // [B*Hq][S][2]   (max in log2 units, sum)
    float* part_acc;                // [B*Hq][S][D]
    int* ghist;                     // [B*Hkv][4096] or nullptr: where a kernel that bins its scores itself adds
                                    // its counts per top-12-bits of the score's ordered key (see topk.hip)
    float* scores;                  // [B*Hkv][score_stride] group-mean scaled scores (second matrix-core
                                    // kernel: nullptr = not wanted)
    int64_t score_stride;           // multiple of 4, >= N
    // self-scheduling mode only.  The wave tiles of a (batch, KV head) (a tile = the rows one
    // wave loads at a time) are cut into n_segs segments of equal length (to within one tile);
    // wgs_per_seg workgroups share a segment.  Chunk c of a segment covers its tiles
    // chunk_tile[c] .. chunk_tile[c + 1] - 1 (the last chunk runs to the segment's end);
    // workgroup w of the segment starts on chunk w, further chunks are claimed from the
    // segment's counter.
    int* chunk_ctr;                 // [B*Hkv][n_segs] counters, kCtrStride ints apart, zero between launches
    int* err_word;                  // pinned host memory (or nullptr): set to 1 if a wave's bounded wait ran out
    int n_segs, wgs_per_seg, total_tiles;
    // Sequences of different lengths (n_segs == 1 only): the workgroups of the launch are
    // dealt out to the (batch, KV head) pairs in proportion to their rows by a small kernel
    // that runs first (ragged_plan.hip).  wg_map[x] for workgroup x of the grid (x counted
    // with the split fastest, then the KV head, then the batch): its pair, its rank w among
    // the pair's n workgroups, the pair's first partial slot and the rows of the pair's
    // sequence; n == 0: nothing to do.
    // nullptr: workgroup x serves pair x / n_splits as number x % n_splits of n_splits.
    const int4* wg_map;             // {pair, w | n << 16, first, rows}
    // Two workgroups share a compute unit, and the one that arrived first streams about 10 %
    // faster (the unit serves its older waves first).  Workgroups are placed in the order of
    // their numbers, so with gen_half = half the grid > 0 the first half of the grid are the
    // early arrivals.  Every group of wgs_per_seg workgroups that shares a chunk counter is then
    // made of wgs_per_seg / 2 workgroups from each half (see paired_unit), so that the groups
    // finish together.  0: workgroup x belongs to group x / wgs_per_seg.
    int gen_half;
    int n_chunks;
    int made_for;                   // = chunk_tile[n_chunks]: the tiles the table was made for (kept beside the
                                    // other scalars: read through the table it would be a second, dependent
                                    // fetch of kernel arguments in front of the first tile's loads)
    int chunk_tile[kMaxChunks + 1];
};

// Merge of the partials + TopK in one launch (topk.hip).
struct TopkParams {
    const float* part_ml;
    const float* part_acc;
    const float* scores;            // [B*Hkv][score_stride] what is ranked: row scores, or block scores
    int64_t score_stride;
    int n_splits, Hq, Hkv, G, D, N, k;
    const int32_t* seq_lens;        // [B] or nullptr: sequence b ranks its first n_b rows and selects
                                    // min(k, n_b) of them; the rest of its k index entries are -1
    int sel_block;                  // rows per ranked unit (N and k count units): n_b = ceil(len / sel_block)
    const int2* pair_map;           // [B*Hkv] {first partial slot, partials} of the pair; nullptr:
                                    // {pair * n_splits, n_splits}.  The pair's partials are laid out
                                    // [head of the group][partial] from slot `first` on (see part_view).
    float* out;                     // [B][Hq][D]
    int32_t* idx;                   // [B][Hkv][k]; nullptr: merge only
    int* ghist;                     // [B*Hkv][4096] histogram of the top 12 key bits of the ranked scores:
                                    // complete when step 0 starts, zero again when step 1 ends
    int2* pair_info;                // [B*Hkv] {level-1 threshold bin, rows in the bins above it}
    int2* chunk_info;               // [B*Hkv][max_chunks] {rows above the threshold bin, rows in it}
    int2* chunk_list;               // [B*Hkv][max_chunks][kTopkChunkList] {key, position} of the rows in it
    int max_chunks;
    uint64_t* headers;              // one-launch form: [B*Hkv][max_chunks][max_chunks] 64-bit {counts, tag} units
                                    // (receiver, sender), all zero between launches; nullptr: not available
    int* err_word;                  // pinned host word set if a bounded wait runs out
    int merge_wgs, merge_lanes;     // workgroups per pair that merge the partials, lanes per output (set by launch_topk)
    int chunks;                     // chunks per (batch, KV head) of this launch (set by launch_topk)
    int64_t pairs;                  // B * Hkv (set by launch_topk)
};
constexpr int kTopkChunkRows = 8192;    // rows of a (batch, KV head) per selecting workgroup
constexpr int kTopkChunkList = 512;     // rows of the level-1 threshold bin a chunk can list
hipError_t launch_score_hist(const TopkParams& p, int B, hipStream_t st);
// step 0: level-1 threshold, per-chunk counts and lists, merge of the partials; step 1: emission;
// step 2: both in one launch (only if topk_one_launch_fits)
hipError_t launch_topk(const TopkParams& p, int B, int step, int n_cus, hipStream_t st);
// Workgroups of the one-launch kernel a compute unit holds at once (a host-side query; 0 on failure).
int topk_one_launch_occupancy();
// Whether every workgroup of the one-launch form would be resident at once (they wait for one another).
bool topk_one_launch_fits(const TopkParams& p, int B, int n_cus, int occupancy);

// Merge by packets (reuse_tail.h): 64-bit units a thread of a consuming workgroup polls at most,
// i.e. a workgroup of T threads receives at most kPacketUnitsPerThread * T units.
constexpr int kPacketUnitsPerThread = 6;

struct ReuseParams {
    const uint16_t* q;
    const uint16_t* K;
    const uint16_t* V;
    int64_t sb, sh, sn;
    RowMap map;
    int Hq, Hkv, N, k;              // k = row slots per (batch, KV head) = idx_stride * block
    int rows_per_split, n_splits;
    float scale_log2;
    const int32_t* idx;             // [B][Hkv][idx_stride]: rows (block == 1) or block numbers
    int idx_stride;                 // entries of idx per (batch, KV head): k / block
    int block;                      // tokens per block; 1 = idx names rows directly
    uint32_t block_magic;           // ceil(2^32 / block), for the division by block
    int n_blocks;                   // ceil(N / block)
    float* part_ml;                 // [B*Hq][S][2]
    float* part_acc;                // [B*Hq][S][D]
    int* counters;                  // [B*Hkv] arrival counters, all zero between launches;
                                    // nullptr: do not merge in this kernel
    float* out;                     // [B][Hq][D], written by the merging workgroup
    // Append-then-attend in one launch (matrix-core kernels only; see reuse_tail.h): the current
    // token's rows [B][Hkv][D], or nullptr.  Then map.seq_lens holds the lengths BEFORE the call
    // (nullptr: N - 1 everywhere) and K, V receive one row per (batch, KV head).
    const uint16_t* k_new;
    const uint16_t* v_new;
    // Merge by packets (reuse_tail.h): [B*Hkv][S][S][units] 64-bit units, all zero between
    // launches, or nullptr: merge by arrival counter.  err_word: pinned host word set if a
    // bounded wait runs out.
    uint64_t* packets;
    int* err_word;
};

// Block-level TopK: scores of blocks of `block` consecutive rows = maximum of the rows' scores.
struct BlockMaxParams {
    const float* scores;            // [B*Hkv][score_stride] row scores
    int64_t score_stride;
    float* bscores;                 // [B*Hkv][bscore_stride] block scores
    int64_t bscore_stride;
    int N, block, n_blocks;
    const int32_t* seq_lens;        // [B] or nullptr: only the blocks that hold rows of sequence b are written
};

// Deal of the Full kernel's workgroups to sequences of different lengths (ragged_plan.hip).
// Per KV head the batch shares S * B workgroups: sequence b gets max(1, ceil(T_b / L)) of them,
// T_b being its wave tiles and L the smallest load per workgroup the S * B workgroups can
// carry; the few left over stay idle.
struct RaggedPlanParams {
    const int32_t* seq_lens;        // [B]
    int B, Hkv, S, N, tile;         // S: workgroups per pair of the launch; tile: rows per wave tile
    int4* wg_map;                   // [B*Hkv*S], see FullParams
    int2* pair_map;                 // [B*Hkv], see FinalizeParams
};
constexpr int kMaxRaggedBatch = 4096;
constexpr int kMaxRaggedWgs = 32767;   // S * B
hipError_t launch_ragged_plan(const RaggedPlanParams& p, hipStream_t st);

// Pooled overlap counts between the index sets of the layers (policy.hip).
constexpr int kMaxProfileLayers = 256;
struct OverlapParams {
    const int32_t* idx[kMaxProfileLayers];   // per layer: [B][Hkv][k]
    int L, Hkv, k, N;
    unsigned long long* counts;               // [L][L]; entries i <= j are written
};

// Index-guided prefetch (offload.hip): selected rows of a (slow) cache into compact buffers.
struct GatherParams {
    const uint16_t* K;              // source cache, addressed through sb / sh / sn (elements), or
    const uint16_t* V;              // through the page table of `map`
    int64_t sb, sh, sn;
    RowMap map;                     // zero: contiguous cache, every sequence N rows
    int Hkv, D, N, k;               // k = row slots per (batch, KV head) = idx_stride * block
    const int32_t* idx;             // [B][Hkv][idx_stride]: rows (block == 1) or block numbers
    int idx_stride, block;
    uint32_t block_magic;           // ceil(2^32 / block)
    int n_blocks;                   // ceil(N / block)
    uint16_t* K_dst;                // [B][Hkv][k][D]
    uint16_t* V_dst;
    int32_t* idx_dst;               // [B][Hkv][k]: the slot's own number, or -1 where it holds no row
};

// Cache update before the attention of a decode step: one new row per (batch, KV head).
struct AppendParams {
    const uint16_t* k_new;          // [B][Hkv][D]
    const uint16_t* v_new;
    uint16_t* K;                    // cache (or pools), addressed like the attention kernels do
    uint16_t* V;
    int64_t sb, sh, sn;
    RowMap map;                     // seq_lens: rows before the call (nullptr: N - 1 everywhere)
    int Hkv, D, N;
    int32_t* lens_out;              // [B] rows after the call, or nullptr
};
hipError_t launch_append_rows(const AppendParams& p, int B, hipStream_t st);

struct CombineParams {
    const float* part_ml;
    const float* part_acc;
    int n_splits, D;
    float* out;                     // [n_heads_total][D]
};

// Rows of the cache one workgroup of the Full kernel consumes per sweep of its 4 waves
// (rows_per_split must be a multiple of it).  0 if (G, variant) is not built.  One pair of
// functions per head_dim, each in its own translation unit.
int full_block_quantum_d64(int G, int variant);
int full_block_quantum_d128(int G, int variant);
hipError_t launch_full_split_d64(const FullParams& p, int B, int G, int variant, hipStream_t st);
hipError_t launch_full_split_d128(const FullParams& p, int B, int G, int variant, hipStream_t st);
// Index entries per workgroup sweep of the Reuse kernel for unroll R in {1, 2, 4, 8}.
int reuse_block_quantum_d64(int G, int variant, int R);
int reuse_block_quantum_d128(int G, int variant, int R);
hipError_t launch_reuse_split_d64(const ReuseParams& p, int B, int G, int variant, int R, hipStream_t st);
hipError_t launch_reuse_split_d128(const ReuseParams& p, int B, int G, int variant, int R, hipStream_t st);

// Matrix-core Full kernel (full_mfma.hip): variant 52
int full_mfma_quantum(int variant);
hipError_t launch_full_mfma(const FullParams& p, int B, int D, int G, int variant, hipStream_t st);

// Second matrix-core Full kernel (full_mfma2.hip; head_dim 128): variant 72
int full_mfma2_quantum(int D, int variant);
hipError_t launch_full_mfma2(const FullParams& p, int B, int G, int variant, hipStream_t st);

inline int full_block_quantum(int D, int G, int variant) {
    if (variant >= 70) return full_mfma2_quantum(D, variant);
    if (variant >= 50) return (D == 64 || D == 128) ? full_mfma_quantum(variant) : 0;
    return D == 64 ? full_block_quantum_d64(G, variant) : D == 128 ? full_block_quantum_d128(G, variant) : 0;
}
inline hipError_t launch_full_split(const FullParams& p, int B, int D, int G, int variant, hipStream_t st) {
    if (variant >= 70) return D == 128 ? launch_full_mfma2(p, B, G, variant, st) : hipErrorInvalidValue;
    if (variant >= 50) return launch_full_mfma(p, B, D, G, variant, st);
    return D == 64 ? launch_full_split_d64(p, B, G, variant, st)
         : D == 128 ? launch_full_split_d128(p, B, G, variant, st) : hipErrorInvalidValue;
}
inline int reuse_block_quantum(int D, int G, int variant, int R) {
    return D == 64 ? reuse_block_quantum_d64(G, variant, R) : D == 128 ? reuse_block_quantum_d128(G, variant, R) : 0;
}
inline hipError_t launch_reuse_split(const ReuseParams& p, int B, int D, int G, int variant, int R, hipStream_t st) {
    return D == 64 ? launch_reuse_split_d64(p, B, G, variant, R, st)
         : D == 128 ? launch_reuse_split_d128(p, B, G, variant, R, st) : hipErrorInvalidValue;
}

// Matrix-core Reuse kernel: NB blocks of 16 rows per wave tile (1, 2 or 4), NW waves per
// workgroup (4; 8 with NB = 4)
int reuse_mfma_quantum(int NB, int NW);
hipError_t launch_reuse_mfma(const ReuseParams& p, int B, int D, int G, int NB, bool nt, int NW, hipStream_t st);

// Second matrix-core Reuse kernel (head_dim 128): 64 index entries per wave, NW = 4 or 8 waves
int reuse_mfma2_quantum(int D, int NW, int NB);
hipError_t launch_reuse_mfma2(const ReuseParams& p, int B, int G, bool nt, int NW, int NB, hipStream_t st);

hipError_t launch_gather_rows(const GatherParams& p, int B, hipStream_t st);
hipError_t launch_overlap_counts(const OverlapParams& p, int B, hipStream_t st);

hipError_t launch_block_max(const BlockMaxParams& p, int B, int Hkv, hipStream_t st);
hipError_t launch_combine(const CombineParams& p, int n_heads_total, hipStream_t st);
// n ints at p become zero (a kernel: safe to record into a HIP graph)
hipError_t launch_fill_zero(int* p, int n, hipStream_t st);
hipError_t launch_probe_copy(void* dst, const void* src, size_t bytes, hipStream_t st);
hipError_t launch_probe_gather(const GatherParams& p, int B, int n_cus, void* sink, hipStream_t st);
hipError_t launch_probe_read(const void* src, size_t bytes, void* sink, hipStream_t st);

}  // namespace hylra
