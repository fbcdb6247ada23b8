// Host side of libhylra: argument checks, split planning, workspace, launches.
// Nothing here computes attention; every step of the path runs in the kernels.
#include "../../include/hylra.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "launch.h"

using namespace hylra;

namespace {

constexpr int kMaxOffloadLayers = 256;    // layers hylra_decode_step_offloaded accepts (and staging slots it uses)
constexpr int kDynWgsPerSeg = 8;          // workgroups that share a segment in the self-scheduling Full kernel
constexpr int kTargetBlocksFull = 512;    // workgroups the Full kernel aims for: two per CU,
                                          // all resident at once (measured best on MI355X)
constexpr int64_t kMinSlots = 8192;       // partial slots ((batch, KV head, split) triples) kept
constexpr int kMaxBlock = 65536;           // rows per block of the block-level variant
constexpr int kMaxCtx = 1 << 30;
constexpr float LOG2E_HOST = 1.4426950408889634f;

thread_local char g_create_error[256] = "";

// Workspace of hylra_reuse_sparse_attn_static, the entry point that allocates nothing: the
// split partials and arrival counters of the Reuse kernels, laid out as
//   acc  float [kStaticHeadSplits][128]   partial outputs per (query head, split)
//   ml   float [kStaticHeadSplits][2]     their (max, sum)
//   ctr  int   [kStaticPairs]             arrival counter per (batch, KV head)
// Every GPU the library runs on holds its own copy of this array at its own address until the
// process ends.  In host code the array's NAME is only a handle for hipGetSymbolAddress: the
// device address it yields (kept per device in g_scratch_ptr) is what kernels, fills and
// copies are given.
constexpr int64_t kStaticHeadSplits = 4096;
constexpr int64_t kStaticPairs = 2048;
constexpr int64_t kStaticAccBytes = kStaticHeadSplits * 128 * sizeof(float);
constexpr int64_t kStaticMlBytes = kStaticHeadSplits * 2 * sizeof(float);
constexpr int64_t kStaticCtrBytes = kStaticPairs * sizeof(int);
constexpr int64_t kStaticScratchBytes = kStaticAccBytes + kStaticMlBytes + kStaticCtrBytes;
constexpr int kMaxDevices = 64;
}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};
int g_scratch_cus[kMaxDevices] = {};

// Device address of `scratch` on device dev (which must be the current device) and the
// device's compute units; looked up once per device.
hipError_t scratch_on_device(int dev, void** ptr, int* n_cus) {
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        int cus = 0;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        g_scratch_cus[dev] = cus;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    *n_cus = g_scratch_cus[dev];
    return hipSuccess;
}

int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }
int64_t ceil_div(int64_t x, int64_t m) { return (x + m - 1) / m; }

}  // namespace

struct hylra_ctx {
    int device = 0;
    hylra_shape max_shape{};
    int32_t max_k = 0;

    float* part_ml = nullptr;
    float* part_acc = nullptr;
    float* scores = nullptr;
    float* bscores = nullptr;   // block scores of the block-level variant (blocks of >= 2 rows)
    int* counters = nullptr;    // one arrival counter per (batch, KV head), zero between launches
    int* chunk_ctr = nullptr;   // chunk counters of the self-scheduling Full kernel (kCtrStride ints apart)
    int* err_word = nullptr;    // pinned host memory the kernels can write: non-zero = a launch of this context
                                // gave up a bounded wait; its results and the counters cannot be trusted
    int* sel_ws = nullptr;      // selection scratch (see TopkParams and hylra_create_ex)
    int max_chunks = 0;         // chunks of 8192 rows per (batch, KV head) at the maximum context
    int64_t sel_ints = 0;       // ints in sel_ws
    int32_t* lens_plus = nullptr;   // [max batch] sequence lengths after an append (see append_impl)
    uint64_t* packets = nullptr;    // packets of the Reuse kernels' merge (reuse_tail.h), all zero between launches
    int64_t cap_packets = 0;        // 64-bit units
    uint64_t* topk_headers = nullptr;   // [pairs][max_chunks][max_chunks] headers of the one-launch selection, zero between launches
    int64_t n_topk_headers = 0;
    int topk_occupancy = 0;         // workgroups of the one-launch selection a compute unit holds
    int4* wg_map = nullptr;     // deal of the Full kernel's workgroups to sequences of different lengths
    int2* pair_map = nullptr;   // (see RaggedPlanParams): `slots` and `pairs_cap` entries
    int n_cus = 0;              // compute units of the device
    bool in_step = false;       // inside hylra_decode_step*: the lengths are the same for every layer,
    bool step_planned = false;  // so the deal is made once per step
    int64_t pairs_cap = 0;      // (batch, KV head) pairs the selection scratch is sized for
    int64_t slots = 0;          // capacity in (batch, KV head, split) triples
    int64_t cap_acc = 0;        // floats
    int64_t cap_ml = 0;
    int64_t cap_scores = 0;
    int64_t cap_bscores = 0;

    uint32_t flags = 0;         // HYLRA_FLAG_* given at creation

    int32_t opt_full_split_rows = 0;
    int32_t opt_reuse_split_rows = 0;
    int32_t opt_full_variant = 0;
    int32_t opt_reuse_variant = 0;
    int32_t opt_reuse_unroll = 0;
    int32_t opt_reuse_waves = 0;
    int32_t opt_reuse_unfused = 0;
    int32_t opt_ragged_even = 0;
    int32_t opt_full_unpaired = 0;
    int32_t opt_hist_unfused = 0;
    int32_t opt_append_unfused = 0;
    int32_t opt_reuse_merge = 0;
    int32_t opt_topk_two_launches = 0;
    int32_t last_topk_launches = 0;
    int32_t last_reuse_splits = 0, last_reuse_wave_rows = 0, last_reuse_merge = 0;   // see hylra_get_info

    bool prof_on = false;
    int prof_n = 0;
    hipEvent_t* prof_ev = nullptr;          // 2 * HYLRA_PROFILE_MAX_EVENTS, created on first enable
    uint8_t prof_cls[HYLRA_PROFILE_MAX_EVENTS];
    int32_t prof_cnt[HYLRA_PROFILE_MAX_EVENTS];      // launches inside bracket i
    bool prof_open = false;                          // the last bracket still lacks its end event
    hipStream_t prof_stream = nullptr;               // stream of the open bracket

    // index-guided prefetch: events that order the copy stream and the compute stream
    hipEvent_t* off_ev = nullptr;           // [0]: index set ready; [1 .. kMaxOffloadLayers]: layer l gathered;
                                            // then one per staging slot: slot consumed

    mutable char err[256] = "";
};

namespace {

hylra_status fail(const hylra_ctx* ctx, hylra_status s, const char* fmt, ...) {
    char* dst = ctx ? ctx->err : g_create_error;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, 256, fmt, ap);
    va_end(ap);
    return s;
}

#define HIP_TRY(ctx, expr)                                                                  \
    do {                                                                                    \
        hipError_t e_ = (expr);                                                             \
        if (e_ != hipSuccess)                                                               \
            return fail(ctx, HYLRA_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));        \
    } while (0)

struct DeviceGuard {
    int prev = -1;
    bool switched = false;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) == hipSuccess && prev != dev) switched = hipSetDevice(dev) == hipSuccess;
    }
    ~DeviceGuard() {
        if (switched) (void)hipSetDevice(prev);
    }
};

struct Strides {
    int64_t b, h, n;
};

// Shape checks shared by every entry point.  Fills G and the effective strides.
hylra_status check_shape(const hylra_ctx* ctx, const hylra_shape* s, int& G, Strides& st, float& scale) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    if (ctx->err_word && *(volatile int*)ctx->err_word)
        return fail(ctx, HYLRA_ERR_HIP, "an earlier launch of this context gave up waiting (for rows to be handed out, or for another workgroup's partial results): "
                                        "its results are incomplete; call hylra_reset");
    if (!s) return fail(ctx, HYLRA_ERR_BAD_ARG, "shape is NULL");
    if (s->batch < 1 || s->n_q_heads < 1 || s->n_kv_heads < 1 || s->ctx_len < 1)
        return fail(ctx, HYLRA_ERR_BAD_ARG, "batch, head counts and ctx_len must be >= 1");
    if (s->ctx_len > kMaxCtx) return fail(ctx, HYLRA_ERR_UNSUPPORTED, "ctx_len must be <= %d", kMaxCtx);
    if (s->n_q_heads % s->n_kv_heads != 0)
        return fail(ctx, HYLRA_ERR_BAD_ARG, "n_q_heads (%d) is not a multiple of n_kv_heads (%d)",
                    s->n_q_heads, s->n_kv_heads);
    G = s->n_q_heads / s->n_kv_heads;
    if (s->head_dim != 64 && s->head_dim != 128)
        return fail(ctx, HYLRA_ERR_UNSUPPORTED, "head_dim %d: only 64 and 128 are built", s->head_dim);
    if (G > kMaxGroup)
        return fail(ctx, HYLRA_ERR_UNSUPPORTED, "group size %d: at most %d query heads per KV head", G, kMaxGroup);
    if (s->batch > 65535 || s->n_kv_heads > 65535)   // grid.z / grid.y limits
        return fail(ctx, HYLRA_ERR_UNSUPPORTED, "batch and n_kv_heads must each be <= 65535");
    const int D = s->head_dim;
    if (s->kv_stride_b == 0 && s->kv_stride_h == 0 && s->kv_stride_n == 0) {
        st.n = D;
        st.h = (int64_t)s->ctx_len * D;
        st.b = st.h * s->n_kv_heads;
    } else {
        st.b = s->kv_stride_b;
        st.h = s->kv_stride_h;
        st.n = s->kv_stride_n;
        if (st.n < D || st.h < 0 || st.b < 0)
            return fail(ctx, HYLRA_ERR_BAD_ARG, "kv strides must be non-negative and kv_stride_n >= head_dim");
        if (st.n % 8 || st.h % 8 || st.b % 8)
            return fail(ctx, HYLRA_ERR_BAD_ARG, "kv strides must be multiples of 8 elements (16 bytes)");
    }
    if (!(s->scale >= 0.f) || std::isinf(s->scale))
        return fail(ctx, HYLRA_ERR_BAD_ARG, "scale must be finite and >= 0");
    scale = s->scale > 0.f ? s->scale : 1.0f / std::sqrt((float)D);
    return HYLRA_OK;
}

hylra_status check_tensors(const hylra_ctx* ctx, const void* q, const void* K, const void* V, const void* out) {
    if (!q || !K || !V || !out) return fail(ctx, HYLRA_ERR_BAD_ARG, "q, K, V and out must not be NULL");
    if (((uintptr_t)q | (uintptr_t)K | (uintptr_t)V) & 15)
        return fail(ctx, HYLRA_ERR_BAD_ARG, "q, K and V must be 16-byte aligned");
    if ((uintptr_t)out & 3) return fail(ctx, HYLRA_ERR_BAD_ARG, "out must be 4-byte aligned");
    return HYLRA_OK;
}

// Paged cache description -> row map and strides.  pg == nullptr: contiguous cache.
hylra_status check_paged(const hylra_ctx* ctx, const hylra_shape* s, const hylra_paged* pg, Strides& st, RowMap& map) {
    map = RowMap{};
    if (!pg) return HYLRA_OK;
    if (!pg->block_table) {
        // per-sequence lengths over a contiguous cache (addressed through the shape's strides)
        if ((uintptr_t)pg->seq_lens & 3) return fail(ctx, HYLRA_ERR_BAD_ARG, "seq_lens must be 4-byte aligned");
        map.seq_lens = pg->seq_lens;
        return HYLRA_OK;
    }
    if (pg->page_size < 1 || pg->page_size > 65536 || (pg->page_size & (pg->page_size - 1)))
        return fail(ctx, HYLRA_ERR_BAD_ARG, "page_size = %d is not a power of two in 1..65536", pg->page_size);
    if ((int64_t)pg->max_pages * pg->page_size < s->ctx_len)
        return fail(ctx, HYLRA_ERR_BAD_ARG, "max_pages = %d pages of %d rows do not cover ctx_len = %d", pg->max_pages, pg->page_size, s->ctx_len);
    if (((uintptr_t)pg->block_table & 3) || ((uintptr_t)pg->seq_lens & 3))
        return fail(ctx, HYLRA_ERR_BAD_ARG, "block_table and seq_lens must be 4-byte aligned device pointers");
    if (pg->stride_row < s->head_dim || pg->stride_head < 0 || pg->stride_page < 0)
        return fail(ctx, HYLRA_ERR_BAD_ARG, "pool strides must be non-negative and stride_row >= head_dim");
    if (pg->stride_row % 8 || pg->stride_head % 8 || pg->stride_page % 8)
        return fail(ctx, HYLRA_ERR_BAD_ARG, "pool strides must be multiples of 8 elements (16 bytes)");
    st.b = 0, st.h = pg->stride_head, st.n = pg->stride_row;
    map.table = pg->block_table;
    map.seq_lens = pg->seq_lens;
    map.table_stride = pg->max_pages;
    map.page_shift = 0;
    while ((1 << map.page_shift) < pg->page_size) ++map.page_shift;
    map.stride_page = pg->stride_page;
    return HYLRA_OK;
}

// Page-table entries a workgroup that touches `rows` consecutive rows may have to stage in
// LDS, given that `other_lds` bytes of dynamic LDS are taken already; 0 (= look the table up
// in memory) if that would not fit.
int table_capacity(const RowMap& map, int64_t rows, int64_t other_lds) {
    if (!map.table) return 0;
    const int64_t n = (rows >> map.page_shift) + 3;
    return other_lds + n * 4 <= 48 * 1024 ? (int)n : 0;
}

// Ends the open event bracket, if any, on the stream it was opened on.
hipError_t close_bracket(hylra_ctx* ctx) {
    if (!ctx->prof_open) return hipSuccess;
    ctx->prof_open = false;
    return hipEventRecord(ctx->prof_ev[2 * (ctx->prof_n - 1) + 1], ctx->prof_stream);
}

// Runs a launch, timed by events when profiling is on.  Consecutive launches of one class on
// one stream share a bracket (start event before the first, end event after the last): the
// events then cost nothing between the launches, and the bracket's time divided by its
// launches is what one launch costs back to back, gaps included.
template <class F>
hipError_t launch_timed(hylra_ctx* ctx, int cls, hipStream_t st, F&& f) {
    if (!ctx->prof_on) return f();
    if (ctx->prof_open && ctx->prof_cls[ctx->prof_n - 1] == cls && ctx->prof_stream == st) {
        ++ctx->prof_cnt[ctx->prof_n - 1];
        return f();
    }
    hipError_t e = close_bracket(ctx);
    if (e != hipSuccess) return e;
    if (ctx->prof_n >= HYLRA_PROFILE_MAX_EVENTS) return f();
    const int n = ctx->prof_n;
    e = hipEventRecord(ctx->prof_ev[2 * n], st);
    if (e != hipSuccess) return e;
    e = f();
    if (e != hipSuccess) return e;
    ctx->prof_cls[n] = (uint8_t)cls;
    ctx->prof_cnt[n] = 1;
    ctx->prof_n = n + 1;
    ctx->prof_open = true;
    ctx->prof_stream = st;
    return hipSuccess;
}

// Full kernels that hand out rows at run time: 4x (vector) and 74 (matrix cores)
bool is_self_scheduling(int variant) { return variant / 10 == 4 || variant == 74; }

struct FullPlan {
    int rows_per_split, n_splits, variant;
    int n_segs, wgs_per_seg;        // self-scheduling kernel: n_splits = n_segs * wgs_per_seg
};

// Workgroups per (batch, KV head) of a self-scheduling Full kernel whose wave tile has `tile`
// rows, and the segments they form.  Only the number of workgroups is planned (rows are handed
// out at run time); "full_split_rows" still sets it, as ctx_len / rows.  More than
// kDynWgsPerSeg workgroups per pair are put into equal segments of at most that many: the
// workgroups of a segment then sit on different XCDs and the chunk table stays short.
void plan_dyn_groups(const hylra_ctx* ctx, const hylra_shape* s, int64_t tile, int64_t& S, int64_t& segs) {
    const int64_t pairs = (int64_t)s->batch * s->n_kv_heads;
    const int64_t tiles = ceil_div(s->ctx_len, tile);
    // never more workgroups than are resident at once (two per compute unit): one that has to
    // wait for a place starts on its first chunk when the others are nearly done
    // (batch 12 / 20K: 186 us with 576 workgroups, 157 us with 480)
    S = ctx->opt_full_split_rows > 0 ? ceil_div(s->ctx_len, ctx->opt_full_split_rows)
                                     : std::max<int64_t>(1, kTargetBlocksFull / pairs);
    if (S > ceil_div(tiles, 4)) S = ceil_div(tiles, 4);
    if (S > kMaxSplits) S = kMaxSplits;
    while (S > 1 && pairs * S > ctx->slots) --S;
    segs = ceil_div(S, kDynWgsPerSeg);
    S = segs * (S / segs);
}

// Exactly two workgroups per compute unit and groups of an even number of workgroups: every
// group of a self-scheduling kernel can then be made of early and late arrivals on the
// compute units in equal parts (FullParams::gen_half).
bool pairs_generations(const hylra_ctx* ctx, const hylra_shape* s, int64_t S, int64_t segs) {
    const int64_t grid = (int64_t)s->batch * s->n_kv_heads * S;
    return grid == 2 * (int64_t)ctx->n_cus && (S / segs) % 2 == 0 && !ctx->opt_full_unpaired;
}

hylra_status plan_full(const hylra_ctx* ctx, const hylra_shape* s, int G, FullPlan& pl) {
    // automatic (measured on the benchmark shapes).  head_dim 128: the second matrix-core
    // kernel.  Self-scheduling while a (batch, KV head) gets at most one segment of workgroups
    // (2 % faster than the self-scheduling vector kernel at batch 8 / 32K, equal at batch 32 /
    // 16K; up to 4 heads per group) or whenever its groups can mix early and late workgroups
    // (then also 1 .. 2 % ahead of the even split at batch 1 / 131K and at G = 7); evenly split
    // otherwise (batch 3 / 50K: 98 us against 101 us for the vector kernel and for the
    // self-scheduling form without mixing) and for small problems (under 2048 rows per workgroup).
    // head_dim 64: the vector kernels up to 4 heads per group, the first matrix-core kernel above.
    const int64_t pairs = (int64_t)s->batch * s->n_kv_heads;
    const bool one_segment = kTargetBlocksFull / pairs <= kDynWgsPerSeg;
    bool mixes = false, small = false;
    if (s->head_dim == 128) {
        int64_t S, segs;
        plan_dyn_groups(ctx, s, full_block_quantum(128, G, 74) / 4, S, segs);
        mixes = pairs_generations(ctx, s, S, segs);
        // below about 2048 rows per workgroup the run-time hand-out costs more at the start than
        // it balances (batch 1 / 32K: 33 us against 27.5 us evenly split; batch 8 / 8K: 52 vs 48.5)
        small = s->ctx_len / S < 2048;
    }
    const bool fixed_order = (ctx->flags & HYLRA_FLAG_DETERMINISTIC) != 0;     // no run-time hand-out of rows
    pl.variant = ctx->opt_full_variant > 0 ? ctx->opt_full_variant
                 : s->head_dim == 128 ? (small || fixed_order ? 72 : one_segment && G <= 4 ? 74 : mixes ? 74 : 72)
                 : G > 4 ? 52 : one_segment && !fixed_order ? 43 : 23;
    const int quantum = full_block_quantum(s->head_dim, G, pl.variant);
    if (quantum <= 0) return fail(ctx, HYLRA_ERR_UNSUPPORTED, "Full kernel variant %d is not built for d=%d G=%d", pl.variant, s->head_dim, G);
    if (is_self_scheduling(pl.variant)) {
        const int64_t tile = quantum / 4;                      // rows of one wave tile
        int64_t S, segs;
        plan_dyn_groups(ctx, s, tile, S, segs);
        if (pairs * S > ctx->slots)
            return fail(ctx, HYLRA_ERR_WORKSPACE, "batch*n_kv_heads = %lld exceeds the workspace", (long long)pairs);
        // rows of score staging per workgroup: twice its share of the rows, in whole wave tiles
        int64_t stage = round_up(2 * ceil_div(s->ctx_len, S), tile);
        if (stage > kMaxFullSplitRows) stage = kMaxFullSplitRows / tile * tile;
        pl.rows_per_split = (int)stage;
        pl.n_splits = (int)S;
        pl.n_segs = (int)segs;
        pl.wgs_per_seg = (int)(S / segs);
        return HYLRA_OK;
    }
    // (as many splits per pair as keep all workgroups resident at once, see plan_dyn_groups)
    int64_t rps = ctx->opt_full_split_rows > 0 ? ctx->opt_full_split_rows
                                               : ceil_div(s->ctx_len, std::max<int64_t>(1, kTargetBlocksFull / pairs));
    rps = round_up(rps < quantum ? quantum : rps, quantum);
    // the vector kernel stages the scores of its split in LDS
    const bool stages = pl.variant < 50 || pl.variant >= 70;          // kernels that stage the split's scores in LDS
    const int64_t rps_cap = stages ? kMaxFullSplitRows / quantum * quantum : (int64_t)1 << 40;
    if (rps > rps_cap) rps = rps_cap;
    int64_t S = ceil_div(s->ctx_len, rps);
    while ((S > kMaxSplits || pairs * S > ctx->slots) && rps < rps_cap) {
        rps = round_up(rps * 2, quantum);
        if (rps > rps_cap) rps = rps_cap;
        S = ceil_div(s->ctx_len, rps);
        if (S == 1) break;
    }
    if (S > kMaxSplits)
        return fail(ctx, HYLRA_ERR_UNSUPPORTED, "ctx_len = %d needs %lld splits per KV head, at most %d are supported", s->ctx_len, (long long)S, kMaxSplits);
    if (pairs * S > ctx->slots)
        return fail(ctx, HYLRA_ERR_WORKSPACE, "batch*n_kv_heads = %lld exceeds the workspace", (long long)pairs);
    pl.rows_per_split = (int)rps;
    pl.n_splits = (int)S;
    return HYLRA_OK;
}

struct ReusePlan {
    int rows_per_split, n_splits, variant, R, NW;
    bool packets;               // merge by packets instead of by arrival counter (reuse_tail.h)
};

hylra_status plan_reuse(const hylra_ctx* ctx, const hylra_shape* s, int G, int k, ReusePlan& pl) {
    // public ids 1..6 = vector kernel (streaming / plain loads), first matrix-core kernel
    // (streaming / plain loads), second matrix-core kernel (streaming / plain loads).
    // Automatic: the second matrix-core kernel with streaming loads for head_dim 128 (it is
    // built for that only), else the first one with plain loads.
    pl.variant = (ctx->opt_reuse_variant >= 1 && ctx->opt_reuse_variant <= 6) ? ctx->opt_reuse_variant - 1
                 : s->head_dim == 128 ? 4 : 3;
    if (pl.variant >= 4 && s->head_dim != 128) pl.variant -= 2;
    const int64_t pairs = (int64_t)s->batch * s->n_kv_heads;
    // Unroll: 8 row groups per wave tile (64 rows per wave with 8 lanes per row) keeps the
    // whole gather of a layer in flight at once and the number of partials per (batch, KV
    // head) small, which the in-kernel merge needs (its arrival counter serialises).  Smaller
    // tiles only when a single workgroup still covers all k entries.
    pl.R = ctx->opt_reuse_unroll > 0 ? ctx->opt_reuse_unroll : 8;
    const bool mfma = pl.variant >= 2;
    const bool mfma2 = pl.variant >= 4;
    if (mfma2) pl.R = ctx->opt_reuse_unroll == 4 ? 4 : 8;     // (wave tiles of 32 or 64 rows)
    // matrix-core kernels: workgroups of 8 waves when asked for, or when k fills them and there
    // are enough of them for every compute unit (below that, twice as many workgroups of 4
    // waves spread the gather wider: 12.0 instead of 12.7 us at batch 1 / k = 4096)
    pl.NW = 4;
    if (mfma && pl.R == 8 && (ctx->opt_reuse_waves == 8 ||
                              (ctx->opt_reuse_waves == 0 && k >= 512 && k % 512 == 0 && pairs * (k / 512) >= 256)))
        pl.NW = 8;
    auto quantum_of = [&](int R) {
        if (mfma2) return reuse_mfma2_quantum(s->head_dim, pl.NW, R / 2);
        return mfma ? reuse_mfma_quantum(R / 2, pl.NW) : reuse_block_quantum(s->head_dim, G, pl.variant, R);
    };
    while (ctx->opt_reuse_unroll == 0 && !mfma2 && pl.R > (mfma ? 2 : 1) && quantum_of(pl.R / 2) >= k) pl.R /= 2;
    pl.rows_per_split = quantum_of(pl.R);
    if (pl.rows_per_split <= 0)
        return fail(ctx, HYLRA_ERR_UNSUPPORTED, "Reuse kernel variant %d / unroll %d is not built for d=%d G=%d", pl.variant, pl.R, s->head_dim, G);
    int64_t rps = pl.rows_per_split;
    if (ctx->opt_reuse_split_rows > 0) rps = round_up(ctx->opt_reuse_split_rows, pl.rows_per_split);
    // workgroups of 8 waves: one per compute unit is enough to keep the whole gather in flight, so
    // with many (batch, KV head) pairs a workgroup takes more than one sweep and fewer partials
    // cross workgroups (batch 32, k = 1024: one workgroup per pair and no merge, 27.2 vs 29.1 us)
    else if (pl.NW == 8 && ctx->n_cus > 0)
        rps = round_up(ceil_div(pairs * k, ctx->n_cus), pl.rows_per_split);
    int64_t S = ceil_div(k, rps);
    while (S > kMaxSplits || pairs * S > ctx->slots) {
        rps = round_up(rps * 2, pl.rows_per_split);
        S = ceil_div(k, rps);
        if (S == 1) break;
    }
    if (pairs * S > ctx->slots)
        return fail(ctx, HYLRA_ERR_WORKSPACE, "batch*n_kv_heads = %lld exceeds the workspace", (long long)pairs);
    pl.rows_per_split = (int)rps;
    pl.n_splits = (int)S;
    // Merge by packets: second matrix-core kernel, every workgroup resident at once (at most
    // one per compute unit), a power-of-two number of partials that divides the 128 columns,
    // and what a workgroup receives within what its threads poll.  From 8 partials on: with 4
    // the arrival counter is as fast (config 2: 16.1 against 16.5 us), its merging workgroup
    // then loads only 8 KB.
    auto packets_ok = [&](int NW, int64_t n) {
        return mfma2 && ctx->packets && ctx->opt_reuse_unfused == 0 && ctx->opt_reuse_merge != 1 &&
               packets_fit(pairs, n, G, 128, NW * 64, kPacketUnitsPerThread, ctx->n_cus, ctx->cap_packets,
                           ctx->opt_reuse_merge == 2 ? kMergeBlock : 8);
    };
    // With few (batch, KV head) pairs the gather is spread over twice as many workgroups (wave
    // tiles of 32 rows, 128 entries per workgroup) if the packets can carry the merge: the
    // arrival-counter merge by one compute unit does not keep up with that many partials.
    const bool free_choice = ctx->opt_reuse_unroll == 0 && ctx->opt_reuse_waves == 0 && ctx->opt_reuse_split_rows == 0;
    if (mfma2 && free_choice && pl.NW == 4 && k % 128 == 0 && packets_ok(4, k / 128)) {
        pl.R = 4;
        pl.rows_per_split = 128;
        pl.n_splits = k / 128;
    }
    pl.packets = packets_ok(pl.NW, pl.n_splits);
    return HYLRA_OK;
}

hylra_status check_workspace(const hylra_ctx* ctx, const hylra_shape* s, int S, bool need_scores) {
    const int64_t heads = (int64_t)s->batch * s->n_q_heads;
    if (heads * S * s->head_dim > ctx->cap_acc || heads * S * 2 > ctx->cap_ml)
        return fail(ctx, HYLRA_ERR_WORKSPACE, "shape needs %lld partial floats, workspace holds %lld",
                    (long long)(heads * S * s->head_dim), (long long)ctx->cap_acc);
    if (need_scores) {
        const int64_t need = (int64_t)s->batch * s->n_kv_heads * round_up(s->ctx_len, 4);
        if (need > ctx->cap_scores)
            return fail(ctx, HYLRA_ERR_WORKSPACE, "shape needs %lld score floats, workspace holds %lld",
                        (long long)need, (long long)ctx->cap_scores);
    }
    return HYLRA_OK;
}

}  // namespace

extern "C" {

const char* hylra_status_str(hylra_status s) {
    switch (s) {
        case HYLRA_OK: return "ok";
        case HYLRA_ERR_BAD_ARG: return "bad argument";
        case HYLRA_ERR_UNSUPPORTED: return "unsupported shape";
        case HYLRA_ERR_WORKSPACE: return "workspace too small";
        case HYLRA_ERR_POLICY: return "invalid policy";
        case HYLRA_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

const char* hylra_last_error(const hylra_ctx* ctx) { return ctx ? ctx->err : g_create_error; }

hylra_status hylra_create(hylra_ctx** out, const hylra_shape* max_shape, int32_t max_k, int device) {
    return hylra_create_ex(out, max_shape, max_k, device, 0u);
}

hylra_status hylra_create_ex(hylra_ctx** out, const hylra_shape* max_shape, int32_t max_k, int device,
                             uint32_t flags) {
    if (!out) return fail(nullptr, HYLRA_ERR_BAD_ARG, "out is NULL");
    *out = nullptr;
    if (flags & ~(uint32_t)(HYLRA_FLAG_DETERMINISTIC | HYLRA_FLAG_TOPK_EVERY_FULL_LAYER))
        return fail(nullptr, HYLRA_ERR_BAD_ARG, "unknown flag bits 0x%x", flags);
    hylra_ctx* ctx = new (std::nothrow) hylra_ctx;
    if (!ctx) return fail(nullptr, HYLRA_ERR_HIP, "out of host memory");
    int G = 0;
    Strides st{};
    float scale = 0.f;
    hylra_status rc = check_shape(ctx, max_shape, G, st, scale);
    if (rc == HYLRA_OK && (max_k < 1 || max_k > max_shape->ctx_len))
        rc = fail(ctx, HYLRA_ERR_BAD_ARG, "max_k must be in 1..ctx_len");
    int n_dev = 0;
    if (rc == HYLRA_OK && (hipGetDeviceCount(&n_dev) != hipSuccess || device < 0 || device >= n_dev))
        rc = fail(ctx, HYLRA_ERR_HIP, "HIP device %d is not available (%d devices visible)", device, n_dev);
    if (rc != HYLRA_OK) {
        std::memcpy(g_create_error, ctx->err, sizeof g_create_error);
        delete ctx;
        return rc;
    }
    ctx->device = device;
    ctx->flags = flags;
    (void)hipDeviceGetAttribute(&ctx->n_cus, hipDeviceAttributeMultiprocessorCount, device);
    ctx->max_shape = *max_shape;
    ctx->max_k = max_k;
    const int64_t pairs = (int64_t)max_shape->batch * max_shape->n_kv_heads;
    // enough partial slots for the Full kernel's smallest split count at the maximum context
    const int64_t min_splits = ceil_div(max_shape->ctx_len, kMaxFullSplitRows - 256);
    ctx->slots = pairs * (min_splits > 2 ? min_splits : 2);
    if (ctx->slots < kMinSlots) ctx->slots = kMinSlots;
    ctx->cap_acc = ctx->slots * G * max_shape->head_dim;
    ctx->cap_ml = ctx->slots * G * 2;
    ctx->cap_scores = pairs * round_up(max_shape->ctx_len, 4);
    ctx->cap_bscores = pairs * round_up(ceil_div(max_shape->ctx_len, 2), 4);

    DeviceGuard guard(device);
    hipError_t e = hipMalloc((void**)&ctx->part_acc, ctx->cap_acc * sizeof(float));
    if (e == hipSuccess) e = hipMalloc((void**)&ctx->part_ml, ctx->cap_ml * sizeof(float));
    if (e == hipSuccess) e = hipMalloc((void**)&ctx->scores, ctx->cap_scores * sizeof(float));
    if (e == hipSuccess) e = hipMalloc((void**)&ctx->bscores, ctx->cap_bscores * sizeof(float));
    if (e == hipSuccess) e = hipMalloc((void**)&ctx->counters, ctx->slots * sizeof(int));
    if (e == hipSuccess) e = hipMemset(ctx->counters, 0, ctx->slots * sizeof(int));
    ctx->pairs_cap = pairs;
    // selection scratch (see TopkParams): level-1 histograms; threshold per pair; per chunk of
    // 8192 rows its counts and its list of rows in the threshold bin
    ctx->max_chunks = (int)ceil_div(max_shape->ctx_len, kTopkChunkRows);
    const int64_t sel_ints = pairs * (4096 + 2 + (int64_t)ctx->max_chunks * (2 + 2 * kTopkChunkList));
    ctx->sel_ints = sel_ints;
    if (e == hipSuccess) e = hipMalloc((void**)&ctx->sel_ws, sel_ints * sizeof(int));
    if (e == hipSuccess) e = hipMemset(ctx->sel_ws, 0, sel_ints * sizeof(int));
    // one counter per (pair, segment); there are never more segments than partial slots
    if (e == hipSuccess) e = hipMalloc((void**)&ctx->chunk_ctr, ctx->slots * kCtrStride * sizeof(int));
    if (e == hipSuccess) e = hipMemset(ctx->chunk_ctr, 0, ctx->slots * kCtrStride * sizeof(int));
    if (e == hipSuccess) e = hipHostMalloc((void**)&ctx->err_word, 64, hipHostMallocDefault);
    if (e == hipSuccess) *ctx->err_word = 0;
    if (e == hipSuccess) e = hipMalloc((void**)&ctx->wg_map, ctx->slots * sizeof(int4));
    if (e == hipSuccess) e = hipMalloc((void**)&ctx->pair_map, pairs * sizeof(int2));
    if (e == hipSuccess) e = hipMalloc((void**)&ctx->lens_plus, (size_t)max_shape->batch * sizeof(int32_t));
    // packets: used only by launches of at most one workgroup per compute unit, each of which
    // receives at most kPacketUnitsPerThread units per thread
    ctx->cap_packets = (int64_t)std::max(ctx->n_cus, 1) * kPacketUnitsPerThread * 512;
    if (e == hipSuccess) e = hipMalloc((void**)&ctx->packets, ctx->cap_packets * sizeof(uint64_t));
    if (e == hipSuccess) e = hipMemset(ctx->packets, 0, ctx->cap_packets * sizeof(uint64_t));
    // headers of the one-launch selection (left out for contexts whose lengths would need more than 64 MiB of them)
    ctx->n_topk_headers = pairs * ctx->max_chunks * ctx->max_chunks;
    if (ctx->n_topk_headers <= (8 << 20)) {
        if (e == hipSuccess) e = hipMalloc((void**)&ctx->topk_headers, ctx->n_topk_headers * sizeof(uint64_t));
        if (e == hipSuccess) e = hipMemset(ctx->topk_headers, 0, ctx->n_topk_headers * sizeof(uint64_t));
        ctx->topk_occupancy = topk_one_launch_occupancy();
    }
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        fail(nullptr, HYLRA_ERR_HIP, "workspace allocation failed: %s", hipGetErrorString(e));
        hylra_destroy(ctx);
        return HYLRA_ERR_HIP;
    }
    *out = ctx;
    return HYLRA_OK;
}

hylra_status hylra_destroy(hylra_ctx* ctx) {
    if (!ctx) return HYLRA_OK;
    DeviceGuard guard(ctx->device);
    if (ctx->off_ev) {
        for (int i = 0; i < 1 + 2 * kMaxOffloadLayers; ++i)
            if (ctx->off_ev[i]) (void)hipEventDestroy(ctx->off_ev[i]);
        delete[] ctx->off_ev;
    }
    if (ctx->prof_ev) {
        for (int i = 0; i < 2 * HYLRA_PROFILE_MAX_EVENTS; ++i)
            if (ctx->prof_ev[i]) (void)hipEventDestroy(ctx->prof_ev[i]);
        delete[] ctx->prof_ev;
    }
    if (ctx->part_acc) (void)hipFree(ctx->part_acc);
    if (ctx->part_ml) (void)hipFree(ctx->part_ml);
    if (ctx->scores) (void)hipFree(ctx->scores);
    if (ctx->bscores) (void)hipFree(ctx->bscores);
    if (ctx->counters) (void)hipFree(ctx->counters);
    if (ctx->chunk_ctr) (void)hipFree(ctx->chunk_ctr);
    if (ctx->err_word) (void)hipHostFree(ctx->err_word);
    if (ctx->sel_ws) (void)hipFree(ctx->sel_ws);
    if (ctx->wg_map) (void)hipFree(ctx->wg_map);
    if (ctx->pair_map) (void)hipFree(ctx->pair_map);
    if (ctx->lens_plus) (void)hipFree(ctx->lens_plus);
    if (ctx->packets) (void)hipFree(ctx->packets);
    if (ctx->topk_headers) (void)hipFree(ctx->topk_headers);
    delete ctx;
    return HYLRA_OK;
}

hylra_status hylra_reset(hylra_ctx* ctx) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    DeviceGuard guard(ctx->device);
    HIP_TRY(ctx, hipDeviceSynchronize());
    HIP_TRY(ctx, hipMemset(ctx->counters, 0, ctx->slots * sizeof(int)));
    HIP_TRY(ctx, hipMemset(ctx->chunk_ctr, 0, ctx->slots * kCtrStride * sizeof(int)));
    HIP_TRY(ctx, hipMemset(ctx->sel_ws, 0, ctx->sel_ints * sizeof(int)));
    HIP_TRY(ctx, hipMemset(ctx->packets, 0, ctx->cap_packets * sizeof(uint64_t)));
    if (ctx->topk_headers) HIP_TRY(ctx, hipMemset(ctx->topk_headers, 0, ctx->n_topk_headers * sizeof(uint64_t)));
    HIP_TRY(ctx, hipDeviceSynchronize());
    ctx->in_step = false, ctx->step_planned = false;
    if (ctx->err_word) *ctx->err_word = 0;
    return HYLRA_OK;
}

hylra_status hylra_get_info(const hylra_ctx* ctx, const char* name, int32_t* value) {
    if (!ctx || !name || !value) return HYLRA_ERR_BAD_ARG;
    if (!std::strcmp(name, "last_reuse_splits")) *value = ctx->last_reuse_splits;
    else if (!std::strcmp(name, "last_reuse_wave_rows")) *value = ctx->last_reuse_wave_rows;
    else if (!std::strcmp(name, "last_reuse_merge")) *value = ctx->last_reuse_merge;
    else if (!std::strcmp(name, "last_topk_launches")) *value = ctx->last_topk_launches;
    else return HYLRA_ERR_BAD_ARG;
    return HYLRA_OK;
}

hylra_status hylra_set_option(hylra_ctx* ctx, const char* name, int32_t value) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    if (!name || value < 0) return fail(ctx, HYLRA_ERR_BAD_ARG, "option name is NULL or value negative");
    if (!std::strcmp(name, "full_split_rows")) ctx->opt_full_split_rows = value;
    else if (!std::strcmp(name, "reuse_split_rows")) ctx->opt_reuse_split_rows = value;
    else if (!std::strcmp(name, "full_variant")) ctx->opt_full_variant = value;
    else if (!std::strcmp(name, "reuse_variant")) ctx->opt_reuse_variant = value;
    else if (!std::strcmp(name, "reuse_unroll")) ctx->opt_reuse_unroll = value;
    else if (!std::strcmp(name, "reuse_waves")) ctx->opt_reuse_waves = value;
    else if (!std::strcmp(name, "reuse_unfused")) ctx->opt_reuse_unfused = value;
    else if (!std::strcmp(name, "ragged_even")) ctx->opt_ragged_even = value;
    else if (!std::strcmp(name, "full_unpaired")) ctx->opt_full_unpaired = value;
    else if (!std::strcmp(name, "hist_unfused")) ctx->opt_hist_unfused = value;
    else if (!std::strcmp(name, "append_unfused")) ctx->opt_append_unfused = value;
    else if (!std::strcmp(name, "reuse_merge")) ctx->opt_reuse_merge = value;
    else if (!std::strcmp(name, "topk_two_launches")) ctx->opt_topk_two_launches = value;
    else if (!std::strcmp(name, "simulate_give_up")) {      // what a kernel whose bounded wait ran out would report
        if (ctx->err_word) *ctx->err_word = value ? 1 : 0;
    }
    else return fail(ctx, HYLRA_ERR_BAD_ARG, "unknown option '%s'", name);
    return HYLRA_OK;
}

}  // extern "C"

namespace {

hylra_status append_impl(hylra_ctx* ctx, const hylra_shape* shape, const hylra_paged* pg, const void* k_new,
                         const void* v_new, const void* K, const void* V, hylra_paged& eff, const hylra_paged** use,
                         void* hip_stream);
hylra_status check_append_args(hylra_ctx* ctx, const void* k_new, const void* v_new, const void* K, const void* V);

// Full layer.  block == 1: idx receives the k best rows.  block >= 2: idx receives the k best
// blocks of `block` rows (a block scores the maximum of its rows).
// want_idx == false (only from the layer chain): the layer's index set would never be read, so
// only the attention output is produced and idx is left untouched.
hylra_status full_impl(hylra_ctx* ctx, const hylra_shape* shape, const hylra_paged* pg, const void* q,
                       const void* K, const void* V, int32_t block, int32_t k, float* out, int32_t* idx,
                       void* hip_stream, bool want_idx = true) {
    int G = 0;
    Strides sd{};
    float scale = 0.f;
    RowMap map{};
    hylra_status rc = check_shape(ctx, shape, G, sd, scale);
    if (rc != HYLRA_OK) return rc;
    if ((rc = check_paged(ctx, shape, pg, sd, map)) != HYLRA_OK) return rc;
    if ((rc = check_tensors(ctx, q, K, V, out)) != HYLRA_OK) return rc;
    if (!idx || ((uintptr_t)idx & 3)) return fail(ctx, HYLRA_ERR_BAD_ARG, "idx must be a 4-byte aligned device pointer");
    if (block < 1 || block > kMaxBlock) return fail(ctx, HYLRA_ERR_BAD_ARG, "block = %d is outside 1..%d", block, kMaxBlock);
    // what TopK ranks: rows, or blocks of rows
    const int n_sel = (int)ceil_div(shape->ctx_len, block);
    if (k < 1 || k > n_sel)
        return fail(ctx, HYLRA_ERR_BAD_ARG, "k = %d is outside 1..%d (%s)", k, n_sel, block == 1 ? "ctx_len" : "number of blocks");
    if ((int64_t)k * block > round_up(ctx->max_k, block))
        return fail(ctx, HYLRA_ERR_WORKSPACE, "k = %d (x block %d) exceeds the context's max_k = %d", k, block, ctx->max_k);
    FullPlan pl{};
    if ((rc = plan_full(ctx, shape, G, pl)) != HYLRA_OK) return rc;
    if ((rc = check_workspace(ctx, shape, pl.n_splits, true)) != HYLRA_OK) return rc;

    hipStream_t st = (hipStream_t)hip_stream;
    DeviceGuard guard(ctx->device);
    const int2* pair_map = nullptr;
    FullParams fp{};
    fp.q = (const uint16_t*)q;
    fp.K = (const uint16_t*)K;
    fp.V = (const uint16_t*)V;
    fp.sb = sd.b, fp.sh = sd.h, fp.sn = sd.n;
    fp.map = map;
    fp.Hq = shape->n_q_heads, fp.Hkv = shape->n_kv_heads, fp.N = shape->ctx_len;
    fp.rows_per_split = pl.rows_per_split, fp.n_splits = pl.n_splits;
    // rows whose pages one workgroup can touch: its split, or (self-scheduling) its segment
    fp.tbl_cap = table_capacity(map, is_self_scheduling(pl.variant) ? ceil_div(shape->ctx_len, pl.n_segs) + 64 : pl.rows_per_split,
                                pl.variant >= 50 && pl.variant < 70 ? 0 : (int64_t)pl.rows_per_split * 4);
    fp.scale_log2 = scale * LOG2E_HOST;
    fp.scale_mean = scale / (float)G;
    fp.part_ml = ctx->part_ml, fp.part_acc = ctx->part_acc;
    // the vector kernels and the second matrix-core kernel count their scores for the selection
    // themselves (row level; block scores are counted by a launch of their own)
    fp.ghist = want_idx && block == 1 && (pl.variant < 50 || pl.variant >= 70) && !ctx->opt_hist_unfused &&
                       (int64_t)shape->batch * shape->n_kv_heads <= ctx->pairs_cap
                   ? ctx->sel_ws : nullptr;
    // (the second matrix-core kernel leaves the scores out when the layer's index set is not wanted)
    fp.scores = !want_idx && pl.variant >= 70 ? nullptr : ctx->scores;
    fp.score_stride = round_up(shape->ctx_len, 4);
    if (is_self_scheduling(pl.variant)) {
        fp.chunk_ctr = ctx->chunk_ctr;
        fp.err_word = ctx->err_word;
        const int tile = full_block_quantum(shape->head_dim, G, pl.variant) / 4;     // rows of one wave tile
        fp.total_tiles = (int)ceil_div(shape->ctx_len, tile);
        fp.n_segs = pl.n_segs, fp.wgs_per_seg = pl.wgs_per_seg;
        // the table is made for the shortest segment; longer ones (by one tile) extend their last chunk
        fp.n_chunks = make_chunk_table(fp.total_tiles / pl.n_segs, pl.wgs_per_seg, fp.chunk_tile);
        fp.made_for = fp.chunk_tile[fp.n_chunks];
        // exactly two workgroups per compute unit: mix the early and the late ones in every group
        if (pairs_generations(ctx, shape, pl.n_splits, pl.n_segs))
            fp.gen_half = (int)((int64_t)shape->batch * shape->n_kv_heads * pl.n_splits / 2);
        // Sequences of different lengths: the workgroups are dealt out in proportion to the rows
        // (the lengths live on the device, so a small kernel makes the deal; once per decode step).
        if (map.seq_lens && pl.n_segs == 1 && pl.wgs_per_seg > 1 && shape->batch > 1 &&
            shape->batch <= kMaxRaggedBatch && (int64_t)shape->batch * pl.wgs_per_seg <= kMaxRaggedWgs &&
            (int64_t)shape->batch * shape->n_kv_heads <= ctx->pairs_cap &&
            !ctx->opt_ragged_even) {
            if (!(ctx->in_step && ctx->step_planned)) {
                RaggedPlanParams gp{};
                gp.seq_lens = map.seq_lens;
                gp.B = shape->batch, gp.Hkv = shape->n_kv_heads, gp.S = pl.wgs_per_seg;
                gp.N = shape->ctx_len, gp.tile = tile;
                gp.wg_map = ctx->wg_map, gp.pair_map = ctx->pair_map;
                HIP_TRY(ctx, close_bracket(ctx));                // (the deal belongs to no profiling class)
                HIP_TRY(ctx, launch_ragged_plan(gp, st));
                ctx->step_planned = true;
            }
            fp.wg_map = ctx->wg_map;
            pair_map = ctx->pair_map;
        }
    }
    HIP_TRY(ctx, launch_timed(ctx, 0, st, [&] {
                return launch_full_split(fp, shape->batch, shape->head_dim, G, pl.variant, st);
            }));

    const int64_t pairs = (int64_t)shape->batch * shape->n_kv_heads;
    const bool hist_in_kernel = fp.ghist != nullptr;
    const float* sel_scores = ctx->scores;
    int64_t sel_stride = fp.score_stride;
    if (block > 1 && want_idx) {
        BlockMaxParams bp{};
        bp.scores = ctx->scores, bp.score_stride = fp.score_stride;
        bp.bscores = ctx->bscores, bp.bscore_stride = round_up(n_sel, 4);
        bp.N = shape->ctx_len, bp.block = block, bp.n_blocks = n_sel;
        bp.seq_lens = map.seq_lens;
        if (pairs * bp.bscore_stride > ctx->cap_bscores)
            return fail(ctx, HYLRA_ERR_WORKSPACE, "shape needs %lld block-score floats, workspace holds %lld",
                        (long long)(pairs * bp.bscore_stride), (long long)ctx->cap_bscores);
        HIP_TRY(ctx, launch_timed(ctx, 1, st, [&] { return launch_block_max(bp, shape->batch, shape->n_kv_heads, st); }));
        sel_scores = ctx->bscores;
        sel_stride = bp.bscore_stride;
    }
    // Merge of the partials and TopK: one launch, several workgroups per (batch, KV head).
    // Its level-1 histogram comes from the streaming kernel where that bins its scores
    // itself, else from a small launch in front.
    if (pairs > ctx->pairs_cap)
        return fail(ctx, HYLRA_ERR_WORKSPACE, "batch*n_kv_heads = %lld exceeds the selection workspace", (long long)pairs);
    TopkParams tp{};
    tp.part_ml = ctx->part_ml, tp.part_acc = ctx->part_acc;
    tp.scores = sel_scores, tp.score_stride = sel_stride;
    tp.n_splits = pl.n_splits, tp.Hq = shape->n_q_heads, tp.Hkv = shape->n_kv_heads;
    tp.G = G, tp.D = shape->head_dim, tp.N = n_sel, tp.k = k;
    tp.seq_lens = map.seq_lens, tp.sel_block = block;
    tp.pair_map = pair_map;
    tp.out = out, tp.idx = want_idx ? idx : nullptr;
    tp.ghist = ctx->sel_ws;
    tp.pair_info = reinterpret_cast<int2*>(ctx->sel_ws + ctx->pairs_cap * 4096);
    tp.chunk_info = tp.pair_info + ctx->pairs_cap;
    tp.chunk_list = tp.chunk_info + ctx->pairs_cap * ctx->max_chunks;
    tp.max_chunks = ctx->max_chunks;
    tp.headers = ctx->topk_headers, tp.err_word = ctx->err_word;
    if (want_idx && ceil_div(n_sel, kTopkChunkRows) > ctx->max_chunks)
        return fail(ctx, HYLRA_ERR_WORKSPACE, "ctx_len = %d exceeds the selection workspace", shape->ctx_len);
    if (want_idx && !hist_in_kernel)
        HIP_TRY(ctx, launch_timed(ctx, 1, st, [&] { return launch_score_hist(tp, shape->batch, st); }));
    // The selection in one launch when all its workgroups are resident at once (they wait for
    // one another's counts), else in two.
    const bool one = want_idx && ctx->opt_topk_two_launches == 0 &&
                     topk_one_launch_fits(tp, shape->batch, ctx->n_cus, ctx->topk_occupancy);
    ctx->last_topk_launches = !want_idx ? 0 : one ? 1 : 2;
    if (one) {
        HIP_TRY(ctx, launch_timed(ctx, 1, st, [&] { return launch_topk(tp, shape->batch, 2, ctx->n_cus, st); }));
        return HYLRA_OK;
    }
    for (int step = 0; step < (want_idx ? 2 : 1); ++step)
        HIP_TRY(ctx, launch_timed(ctx, 1, st, [&] { return launch_topk(tp, shape->batch, step, ctx->n_cus, st); }));
    return HYLRA_OK;
}

// Reuse layer over n_idx inherited entries per (batch, KV head): rows (block == 1) or blocks.
hylra_status reuse_impl(hylra_ctx* ctx, const hylra_shape* shape, const hylra_paged* pg, const void* q,
                        const void* K, const void* V, const int32_t* idx, int32_t block, int32_t n_idx,
                        float* out, void* hip_stream, bool clear_counters = false, const void* k_new = nullptr,
                        const void* v_new = nullptr) {
    int G = 0;
    Strides sd{};
    float scale = 0.f;
    RowMap map{};
    hylra_status rc = check_shape(ctx, shape, G, sd, scale);
    if (rc != HYLRA_OK) return rc;
    if ((rc = check_paged(ctx, shape, pg, sd, map)) != HYLRA_OK) return rc;
    if ((rc = check_tensors(ctx, q, K, V, out)) != HYLRA_OK) return rc;
    if (!idx || ((uintptr_t)idx & 3)) return fail(ctx, HYLRA_ERR_BAD_ARG, "idx must be a 4-byte aligned device pointer");
    if (block < 1 || block > kMaxBlock) return fail(ctx, HYLRA_ERR_BAD_ARG, "block = %d is outside 1..%d", block, kMaxBlock);
    if (n_idx < 1) return fail(ctx, HYLRA_ERR_BAD_ARG, "k = %d must be >= 1", n_idx);
    if ((int64_t)n_idx * block > round_up(ctx->max_k, block))
        return fail(ctx, HYLRA_ERR_WORKSPACE, "k = %d (x block %d) exceeds the context's max_k = %d", n_idx, block, ctx->max_k);
    const int k = n_idx * block;            // row slots; fits: max_k <= ctx_len < 2^31 - block is checked at create
    ReusePlan pl{};
    if ((rc = plan_reuse(ctx, shape, G, k, pl)) != HYLRA_OK) return rc;
    if ((rc = check_workspace(ctx, shape, pl.n_splits, false)) != HYLRA_OK) return rc;
    // k_new: the current token's rows go into the cache first.  The matrix-core kernels do that
    // themselves (pg's lengths are then those before the call); for the vector kernel a launch of
    // its own writes the rows and the "length + 1" array the attention then uses.
    const bool append_fused = k_new && pl.variant >= 2 && ctx->opt_append_unfused == 0;
    if (k_new && !append_fused) {
        hylra_paged eff{};
        const hylra_paged* use = nullptr;
        if ((rc = append_impl(ctx, shape, pg, k_new, v_new, K, V, eff, &use, hip_stream)) != HYLRA_OK) return rc;
        if (use && use->seq_lens) map.seq_lens = use->seq_lens;
    }
    if (append_fused && (rc = check_append_args(ctx, k_new, v_new, K, V)) != HYLRA_OK) return rc;

    hipStream_t st = (hipStream_t)hip_stream;
    DeviceGuard guard(ctx->device);
    ReuseParams rp{};
    if (append_fused) rp.k_new = (const uint16_t*)k_new, rp.v_new = (const uint16_t*)v_new;
    rp.q = (const uint16_t*)q;
    rp.K = (const uint16_t*)K;
    rp.V = (const uint16_t*)V;
    rp.sb = sd.b, rp.sh = sd.h, rp.sn = sd.n;
    rp.map = map;
    rp.Hq = shape->n_q_heads, rp.Hkv = shape->n_kv_heads, rp.N = shape->ctx_len, rp.k = k;
    rp.rows_per_split = pl.rows_per_split, rp.n_splits = pl.n_splits;
    rp.scale_log2 = scale * LOG2E_HOST;
    rp.idx = idx;
    rp.idx_stride = n_idx, rp.block = block;
    rp.block_magic = block > 1 ? (uint32_t)((0x100000000ull + (uint32_t)block - 1) / (uint32_t)block) : 0u;
    rp.n_blocks = (int)ceil_div(shape->ctx_len, block);
    rp.part_ml = ctx->part_ml, rp.part_acc = ctx->part_acc;
    const bool fused = ctx->opt_reuse_unfused == 0;
    rp.counters = fused ? ctx->counters : nullptr;
    rp.packets = pl.packets ? ctx->packets : nullptr;
    rp.err_word = ctx->err_word;
    ctx->last_reuse_splits = pl.n_splits;
    ctx->last_reuse_wave_rows = pl.variant >= 2 ? 8 * pl.R : 0;
    ctx->last_reuse_merge = !fused ? 0 : pl.n_splits == 1 && pl.variant >= 2 ? 3 : pl.packets ? 2 : 1;
    rp.out = out;
    // (a workspace that other calls may have left in any state: the arrival counters must start
    // at zero; a fill kernel, not a memset, since the caller may be capturing the stream)
    if (clear_counters && fused) HIP_TRY(ctx, launch_fill_zero(ctx->counters, shape->batch * shape->n_kv_heads, st));
    HIP_TRY(ctx, launch_timed(ctx, 2, st, [&] {
                if (pl.variant >= 4)
                    return launch_reuse_mfma2(rp, shape->batch, G, pl.variant == 4, pl.NW, pl.R / 2, st);
                if (pl.variant >= 2)
                    return launch_reuse_mfma(rp, shape->batch, shape->head_dim, G, pl.R / 2, pl.variant == 2, pl.NW, st);
                return launch_reuse_split(rp, shape->batch, shape->head_dim, G, pl.variant, pl.R, st);
            }));
    if (fused) return HYLRA_OK;
    CombineParams cp{};
    cp.part_ml = ctx->part_ml, cp.part_acc = ctx->part_acc;
    cp.n_splits = pl.n_splits, cp.D = shape->head_dim, cp.out = out;
    HIP_TRY(ctx, launch_timed(ctx, 3, st, [&] {
                return launch_combine(cp, shape->batch * shape->n_q_heads, st);
            }));
    return HYLRA_OK;
}

// Algorithm 2 over the layers of one decode step; block == 1 is the token-level form.
hylra_status step_impl(hylra_ctx* ctx, const hylra_shape* shape, const hylra_paged* pg, int32_t n_layers,
                       const uint8_t* policy, const void* const* q_l, const void* const* K_l,
                       const void* const* V_l, int32_t block, int32_t k, float* const* out_l,
                       int32_t* idx_buf, void* hip_stream, const void* const* k_new_l = nullptr,
                       const void* const* v_new_l = nullptr) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    if (n_layers < 1 || !policy || !q_l || !K_l || !V_l || !out_l || !idx_buf)
        return fail(ctx, HYLRA_ERR_BAD_ARG, "n_layers < 1 or a NULL argument");
    if (policy[0] != HYLRA_FULL)
        return fail(ctx, HYLRA_ERR_POLICY, "policy[0] must be Full: layer 0 has no set to inherit");
    for (int l = 0; l < n_layers; ++l) {
        if (policy[l] != HYLRA_FULL && policy[l] != HYLRA_REUSE)
            return fail(ctx, HYLRA_ERR_POLICY, "policy[%d] = %d is neither Full (0) nor Reuse (1)", l, policy[l]);
        if (!q_l[l] || !K_l[l] || !V_l[l] || !out_l[l] || (k_new_l && (!k_new_l[l] || !v_new_l[l])))
            return fail(ctx, HYLRA_ERR_BAD_ARG, "layer %d has a NULL tensor pointer", l);
    }
    // Layers run in order on one stream: a layer's query depends on the previous layer's
    // output in a real model, so nothing here batches across layers.  A Full layer that is
    // followed by another Full layer hands its index set to nobody (a Reuse layer inherits from
    // the most recent Full layer), so its TopK is skipped; the last layer's set is kept because
    // idx_buf is documented to hold the last Full layer's set on return.
    ctx->in_step = true, ctx->step_planned = false;
    hylra_status rc = HYLRA_OK;
    for (int l = 0; l < n_layers && rc == HYLRA_OK; ++l) {
        const bool want_idx = l + 1 == n_layers || policy[l + 1] == HYLRA_REUSE ||
                              (ctx->flags & HYLRA_FLAG_TOPK_EVERY_FULL_LAYER);
        // with new rows: the layer's cache first receives the current token (every layer writes the
        // same "length + 1" array, so the deal of workgroups made at the first layer stays valid)
        // (a Reuse layer takes the rows along in its own launch: see reuse_impl)
        hylra_paged eff{};
        const hylra_paged* use = pg;
        if (k_new_l && policy[l] == HYLRA_FULL &&
            (rc = append_impl(ctx, shape, pg, k_new_l[l], v_new_l[l], K_l[l], V_l[l], eff, &use, hip_stream)) != HYLRA_OK)
            break;
        rc = policy[l] == HYLRA_FULL
                 ? full_impl(ctx, shape, use, q_l[l], K_l[l], V_l[l], block, k, out_l[l], idx_buf, hip_stream, want_idx)
                 : reuse_impl(ctx, shape, pg, q_l[l], K_l[l], V_l[l], idx_buf, block, k, out_l[l], hip_stream, false,
                              k_new_l ? k_new_l[l] : nullptr, k_new_l ? v_new_l[l] : nullptr);
    }
    ctx->in_step = false;
    return rc;
}

}  // namespace

extern "C" {

hylra_status hylra_full_attn_topk(hylra_ctx* ctx, const hylra_shape* shape, const void* q,
                                  const void* K, const void* V, int32_t k, float* out,
                                  int32_t* idx, void* hip_stream) {
    return full_impl(ctx, shape, nullptr, q, K, V, 1, k, out, idx, hip_stream);
}

hylra_status hylra_reuse_sparse_attn(hylra_ctx* ctx, const hylra_shape* shape, const void* q,
                                     const void* K, const void* V, const int32_t* idx, int32_t k,
                                     float* out, void* hip_stream) {
    return reuse_impl(ctx, shape, nullptr, q, K, V, idx, 1, k, out, hip_stream);
}

hylra_status hylra_reuse_sparse_attn_static(const hylra_shape* shape, const void* q, const void* K,
                                            const void* V, const int32_t* idx, int32_t k, float* out,
                                            void* hip_stream) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess)
        return fail(nullptr, HYLRA_ERR_HIP, "no current HIP device");
    void* base = nullptr;
    int n_cus = 0;
    const hipError_t e = scratch_on_device(dev, &base, &n_cus);
    if (e != hipSuccess)
        return fail(nullptr, HYLRA_ERR_HIP, "address of the static workspace on device %d: %s", dev, hipGetErrorString(e));
    if (!shape) return fail(nullptr, HYLRA_ERR_BAD_ARG, "shape is NULL");
    // a context that owns nothing: its workspace pointers name parts of the static array
    hylra_ctx tmp;
    tmp.device = dev;
    tmp.n_cus = n_cus;
    tmp.max_shape = *shape;
    tmp.max_k = k;
    char* b = static_cast<char*>(base);
    tmp.part_acc = reinterpret_cast<float*>(b);
    tmp.part_ml = reinterpret_cast<float*>(b + kStaticAccBytes);
    tmp.counters = reinterpret_cast<int*>(b + kStaticAccBytes + kStaticMlBytes);
    tmp.slots = kStaticPairs;
    tmp.cap_acc = kStaticHeadSplits * 128;
    tmp.cap_ml = kStaticHeadSplits * 2;
    hylra_status rc = HYLRA_OK;
    const int64_t pairs = (int64_t)shape->batch * shape->n_kv_heads;
    if (shape->batch < 1 || shape->n_kv_heads < 1 || pairs > kStaticPairs)
        rc = fail(&tmp, HYLRA_ERR_WORKSPACE, "batch * n_kv_heads = %lld exceeds the static workspace's %lld pairs",
                  (long long)pairs, (long long)kStaticPairs);
    // the array keeps what the last call left, so reuse_impl clears the counters it will use
    if (rc == HYLRA_OK) rc = reuse_impl(&tmp, shape, nullptr, q, K, V, idx, 1, k, out, hip_stream, true);
    if (rc != HYLRA_OK) std::memcpy(g_create_error, tmp.err, sizeof g_create_error);
    return rc;
}

hylra_status hylra_decode_step(hylra_ctx* ctx, const hylra_shape* shape, int32_t n_layers,
                               const uint8_t* policy, const void* const* q_l,
                               const void* const* K_l, const void* const* V_l, int32_t k,
                               float* const* out_l, int32_t* idx_buf, void* hip_stream) {
    return step_impl(ctx, shape, nullptr, n_layers, policy, q_l, K_l, V_l, 1, k, out_l, idx_buf, hip_stream);
}

hylra_status hylra_full_attn_topk_blocks(hylra_ctx* ctx, const hylra_shape* shape, const void* q,
                                         const void* K, const void* V, int32_t block, int32_t kb,
                                         float* out, int32_t* bidx, void* hip_stream) {
    return full_impl(ctx, shape, nullptr, q, K, V, block, kb, out, bidx, hip_stream);
}

hylra_status hylra_reuse_block_attn(hylra_ctx* ctx, const hylra_shape* shape, const void* q,
                                    const void* K, const void* V, const int32_t* bidx,
                                    int32_t block, int32_t kb, float* out, void* hip_stream) {
    return reuse_impl(ctx, shape, nullptr, q, K, V, bidx, block, kb, out, hip_stream);
}

hylra_status hylra_decode_step_blocks(hylra_ctx* ctx, const hylra_shape* shape, int32_t n_layers,
                                      const uint8_t* policy, const void* const* q_l,
                                      const void* const* K_l, const void* const* V_l, int32_t block,
                                      int32_t kb, float* const* out_l, int32_t* bidx_buf,
                                      void* hip_stream) {
    return step_impl(ctx, shape, nullptr, n_layers, policy, q_l, K_l, V_l, block, kb, out_l, bidx_buf, hip_stream);
}

hylra_status hylra_full_attn_topk_paged(hylra_ctx* ctx, const hylra_shape* shape, const hylra_paged* cache,
                                        const void* q, const void* K_pool, const void* V_pool, int32_t k,
                                        float* out, int32_t* idx, void* hip_stream) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    if (!cache) return fail(ctx, HYLRA_ERR_BAD_ARG, "cache is NULL");
    return full_impl(ctx, shape, cache, q, K_pool, V_pool, 1, k, out, idx, hip_stream);
}

hylra_status hylra_reuse_sparse_attn_paged(hylra_ctx* ctx, const hylra_shape* shape, const hylra_paged* cache,
                                           const void* q, const void* K_pool, const void* V_pool,
                                           const int32_t* idx, int32_t k, float* out, void* hip_stream) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    if (!cache) return fail(ctx, HYLRA_ERR_BAD_ARG, "cache is NULL");
    return reuse_impl(ctx, shape, cache, q, K_pool, V_pool, idx, 1, k, out, hip_stream);
}

hylra_status hylra_decode_step_paged(hylra_ctx* ctx, const hylra_shape* shape, const hylra_paged* cache,
                                     int32_t n_layers, const uint8_t* policy, const void* const* q_l,
                                     const void* const* K_pool_l, const void* const* V_pool_l, int32_t k,
                                     float* const* out_l, int32_t* idx_buf, void* hip_stream) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    if (!cache) return fail(ctx, HYLRA_ERR_BAD_ARG, "cache is NULL");
    return step_impl(ctx, shape, cache, n_layers, policy, q_l, K_pool_l, V_pool_l, 1, k, out_l, idx_buf, hip_stream);
}

hylra_status hylra_full_attn_topk_blocks_paged(hylra_ctx* ctx, const hylra_shape* shape, const hylra_paged* cache,
                                               const void* q, const void* K_pool, const void* V_pool,
                                               int32_t block, int32_t kb, float* out, int32_t* bidx,
                                               void* hip_stream) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    if (!cache) return fail(ctx, HYLRA_ERR_BAD_ARG, "cache is NULL");
    return full_impl(ctx, shape, cache, q, K_pool, V_pool, block, kb, out, bidx, hip_stream);
}

hylra_status hylra_reuse_block_attn_paged(hylra_ctx* ctx, const hylra_shape* shape, const hylra_paged* cache,
                                          const void* q, const void* K_pool, const void* V_pool,
                                          const int32_t* bidx, int32_t block, int32_t kb, float* out,
                                          void* hip_stream) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    if (!cache) return fail(ctx, HYLRA_ERR_BAD_ARG, "cache is NULL");
    return reuse_impl(ctx, shape, cache, q, K_pool, V_pool, bidx, block, kb, out, hip_stream);
}

hylra_status hylra_decode_step_blocks_paged(hylra_ctx* ctx, const hylra_shape* shape, const hylra_paged* cache,
                                            int32_t n_layers, const uint8_t* policy, const void* const* q_l,
                                            const void* const* K_pool_l, const void* const* V_pool_l,
                                            int32_t block, int32_t kb, float* const* out_l, int32_t* bidx_buf,
                                            void* hip_stream) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    if (!cache) return fail(ctx, HYLRA_ERR_BAD_ARG, "cache is NULL");
    return step_impl(ctx, shape, cache, n_layers, policy, q_l, K_pool_l, V_pool_l, block, kb, out_l, bidx_buf, hip_stream);
}

size_t hylra_offload_slot_bytes(const hylra_shape* shape, int32_t k) {
    if (!shape || k < 1 || shape->batch < 1 || shape->n_kv_heads < 1 || shape->head_dim < 1) return 0;
    const size_t rows = (size_t)shape->batch * shape->n_kv_heads * (size_t)k;
    const size_t kv = (rows * shape->head_dim * 2 + 255) / 256 * 256;          // one of K, V (bf16)
    return 2 * kv + (rows * 4 + 255) / 256 * 256;
}

namespace {
struct Slot {
    void* K;
    void* V;
    int32_t* idx;
};
Slot slot_at(void* staging, const hylra_shape* shape, int32_t k, int i) {
    const size_t rows = (size_t)shape->batch * shape->n_kv_heads * (size_t)k;
    const size_t kv = (rows * shape->head_dim * 2 + 255) / 256 * 256;
    char* base = (char*)staging + (size_t)i * hylra_offload_slot_bytes(shape, k);
    return Slot{base, base + kv, (int32_t*)(base + 2 * kv)};
}

// Selected rows (block == 1) or blocks of a cache the device can read into a compact cache of
// n_idx * block rows per (batch, KV head); pg as in the attention calls (nullptr: contiguous).
hylra_status gather_impl(hylra_ctx* ctx, const hylra_shape* shape, const hylra_paged* pg, const void* K_src,
                         const void* V_src, const int32_t* idx, int32_t block, int32_t n_idx, void* K_dst,
                         void* V_dst, int32_t* idx_dst, void* hip_stream) {
    int G = 0;
    Strides sd{};
    float scale = 0.f;
    RowMap map{};
    hylra_status rc = check_shape(ctx, shape, G, sd, scale);
    if (rc != HYLRA_OK) return rc;
    if ((rc = check_paged(ctx, shape, pg, sd, map)) != HYLRA_OK) return rc;
    if (!K_src || !V_src || !idx || !K_dst || !V_dst || !idx_dst)
        return fail(ctx, HYLRA_ERR_BAD_ARG, "a NULL argument");
    if ((((uintptr_t)K_src | (uintptr_t)V_src | (uintptr_t)K_dst | (uintptr_t)V_dst) & 15) ||
        (((uintptr_t)idx | (uintptr_t)idx_dst) & 3))
        return fail(ctx, HYLRA_ERR_BAD_ARG, "caches must be 16-byte aligned, index sets 4-byte aligned");
    if (block < 1 || block > kMaxBlock) return fail(ctx, HYLRA_ERR_BAD_ARG, "block = %d is outside 1..%d", block, kMaxBlock);
    if (n_idx < 1 || (int64_t)n_idx * block > kMaxCtx) return fail(ctx, HYLRA_ERR_BAD_ARG, "k = %d (x block %d) must be in 1..%d", n_idx, block, kMaxCtx);
    GatherParams gp{};
    gp.K = (const uint16_t*)K_src, gp.V = (const uint16_t*)V_src;
    gp.sb = sd.b, gp.sh = sd.h, gp.sn = sd.n;
    gp.map = map;
    gp.Hkv = shape->n_kv_heads, gp.D = shape->head_dim, gp.N = shape->ctx_len, gp.k = n_idx * block;
    gp.idx = idx;
    gp.idx_stride = n_idx, gp.block = block;
    gp.block_magic = block > 1 ? (uint32_t)((0x100000000ull + (uint32_t)block - 1) / (uint32_t)block) : 0u;
    gp.n_blocks = (int)ceil_div(shape->ctx_len, block);
    gp.K_dst = (uint16_t*)K_dst, gp.V_dst = (uint16_t*)V_dst, gp.idx_dst = idx_dst;
    DeviceGuard guard(ctx->device);
    HIP_TRY(ctx, launch_timed(ctx, 3, (hipStream_t)hip_stream, [&] { return launch_gather_rows(gp, shape->batch, (hipStream_t)hip_stream); }));
    return HYLRA_OK;
}

hylra_status check_append_args(hylra_ctx* ctx, const void* k_new, const void* v_new, const void* K, const void* V) {
    if (!k_new || !v_new || !K || !V) return fail(ctx, HYLRA_ERR_BAD_ARG, "k_new, v_new, K and V must not be NULL");
    if (((uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)K | (uintptr_t)V) & 15)
        return fail(ctx, HYLRA_ERR_BAD_ARG, "k_new, v_new, K and V must be 16-byte aligned");
    return HYLRA_OK;
}

// The current token's key / value rows into the cache, behind the rows every sequence has.
// Fills eff (and sets *use) with the cache description the attention that follows must use:
// the caller's, with the lengths replaced by the context's own "length + 1" array.
hylra_status append_impl(hylra_ctx* ctx, const hylra_shape* shape, const hylra_paged* pg, const void* k_new,
                         const void* v_new, const void* K, const void* V, hylra_paged& eff, const hylra_paged** use,
                         void* hip_stream) {
    int G = 0;
    Strides sd{};
    float scale = 0.f;
    RowMap map{};
    hylra_status rc = check_shape(ctx, shape, G, sd, scale);
    if (rc != HYLRA_OK) return rc;
    if ((rc = check_paged(ctx, shape, pg, sd, map)) != HYLRA_OK) return rc;
    if ((rc = check_append_args(ctx, k_new, v_new, K, V)) != HYLRA_OK) return rc;
    if (shape->batch > ctx->max_shape.batch)
        return fail(ctx, HYLRA_ERR_WORKSPACE, "batch = %d exceeds the context's %d", shape->batch, ctx->max_shape.batch);
    AppendParams ap{};
    ap.k_new = (const uint16_t*)k_new, ap.v_new = (const uint16_t*)v_new;
    ap.K = (uint16_t*)K, ap.V = (uint16_t*)V;
    ap.sb = sd.b, ap.sh = sd.h, ap.sn = sd.n;
    ap.map = map;
    ap.Hkv = shape->n_kv_heads, ap.D = shape->head_dim, ap.N = shape->ctx_len;
    ap.lens_out = map.seq_lens ? ctx->lens_plus : nullptr;
    DeviceGuard guard(ctx->device);
    HIP_TRY(ctx, close_bracket(ctx));                    // (belongs to no profiling class)
    HIP_TRY(ctx, launch_append_rows(ap, shape->batch, (hipStream_t)hip_stream));
    *use = pg;
    if (pg && pg->seq_lens) {
        eff = *pg;
        eff.seq_lens = ctx->lens_plus;
        *use = &eff;
    }
    return HYLRA_OK;
}
}  // namespace

hylra_status hylra_gather_rows(hylra_ctx* ctx, const hylra_shape* shape, const void* K_src, const void* V_src,
                               const int32_t* idx, int32_t k, void* K_dst, void* V_dst, int32_t* idx_dst,
                               void* hip_stream) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    return gather_impl(ctx, shape, nullptr, K_src, V_src, idx, 1, k, K_dst, V_dst, idx_dst, hip_stream);
}

hylra_status hylra_gather_blocks(hylra_ctx* ctx, const hylra_shape* shape, const hylra_paged* cache,
                                 const void* K_src, const void* V_src, const int32_t* bidx, int32_t block,
                                 int32_t kb, void* K_dst, void* V_dst, int32_t* idx_dst, void* hip_stream) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    return gather_impl(ctx, shape, cache, K_src, V_src, bidx, block, kb, K_dst, V_dst, idx_dst, hip_stream);
}

hylra_status hylra_append_full_attn_topk(hylra_ctx* ctx, const hylra_shape* shape, const hylra_paged* cache,
                                         const void* q, const void* k_new, const void* v_new, void* K, void* V,
                                         int32_t k, float* out, int32_t* idx, void* hip_stream) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    hylra_paged eff{};
    const hylra_paged* use = nullptr;
    const hylra_status rc = append_impl(ctx, shape, cache, k_new, v_new, K, V, eff, &use, hip_stream);
    if (rc != HYLRA_OK) return rc;
    return full_impl(ctx, shape, use, q, K, V, 1, k, out, idx, hip_stream);
}

hylra_status hylra_append_reuse_sparse_attn(hylra_ctx* ctx, const hylra_shape* shape, const hylra_paged* cache,
                                            const void* q, const void* k_new, const void* v_new, void* K, void* V,
                                            const int32_t* idx, int32_t k, float* out, void* hip_stream) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    if (!k_new || !v_new) return fail(ctx, HYLRA_ERR_BAD_ARG, "k_new, v_new, K and V must not be NULL");
    return reuse_impl(ctx, shape, cache, q, K, V, idx, 1, k, out, hip_stream, false, k_new, v_new);
}

hylra_status hylra_decode_step_append(hylra_ctx* ctx, const hylra_shape* shape, const hylra_paged* cache,
                                      int32_t n_layers, const uint8_t* policy, const void* const* q_l,
                                      const void* const* k_new_l, const void* const* v_new_l, void* const* K_l,
                                      void* const* V_l, int32_t k, float* const* out_l, int32_t* idx_buf,
                                      void* hip_stream) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    if (n_layers < 1 || !k_new_l || !v_new_l || !K_l || !V_l)
        return fail(ctx, HYLRA_ERR_BAD_ARG, "n_layers < 1 or a NULL argument");
    return step_impl(ctx, shape, cache, n_layers, policy, q_l, (const void* const*)K_l, (const void* const*)V_l, 1, k,
                     out_l, idx_buf, hip_stream, k_new_l, v_new_l);
}

namespace {
// Algorithm 2 with the Reuse layers' caches in slow memory: their selected rows (block == 1) or
// blocks are gathered ahead of time on the copy stream; pg as in the attention calls.
hylra_status offloaded_impl(hylra_ctx* ctx, const hylra_shape* shape, const hylra_paged* pg, int32_t n_layers,
                            const uint8_t* policy, const void* const* q_l, const void* const* K_l,
                            const void* const* V_l, int32_t block, int32_t k, float* const* out_l, int32_t* idx_buf,
                            void* staging, size_t staging_bytes, void* compute_stream, void* copy_stream) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    if (n_layers < 1 || !policy || !q_l || !K_l || !V_l || !out_l || !idx_buf || !staging || !shape)
        return fail(ctx, HYLRA_ERR_BAD_ARG, "n_layers < 1 or a NULL argument");
    if (n_layers > kMaxOffloadLayers) return fail(ctx, HYLRA_ERR_UNSUPPORTED, "at most %d layers", kMaxOffloadLayers);
    if (policy[0] != HYLRA_FULL)
        return fail(ctx, HYLRA_ERR_POLICY, "policy[0] must be Full: layer 0 has no set to inherit");
    for (int l = 0; l < n_layers; ++l) {
        if (policy[l] != HYLRA_FULL && policy[l] != HYLRA_REUSE)
            return fail(ctx, HYLRA_ERR_POLICY, "policy[%d] = %d is neither Full (0) nor Reuse (1)", l, policy[l]);
        if (!q_l[l] || !K_l[l] || !V_l[l] || !out_l[l])
            return fail(ctx, HYLRA_ERR_BAD_ARG, "layer %d has a NULL tensor pointer", l);
    }
    if ((uintptr_t)staging & 255) return fail(ctx, HYLRA_ERR_BAD_ARG, "staging must be 256-byte aligned");
    if (block < 1 || block > kMaxBlock) return fail(ctx, HYLRA_ERR_BAD_ARG, "block = %d is outside 1..%d", block, kMaxBlock);
    if (k < 1 || (int64_t)k * block > ctx->max_k)
        return fail(ctx, k < 1 ? HYLRA_ERR_BAD_ARG : HYLRA_ERR_WORKSPACE, "k = %d (x block %d) is outside 1..max_k = %d", k, block, ctx->max_k);
    const int32_t rows = k * block;                     // rows of a compacted cache
    const size_t slot_bytes = hylra_offload_slot_bytes(shape, rows);
    if (slot_bytes == 0 || staging_bytes < slot_bytes)
        return fail(ctx, HYLRA_ERR_WORKSPACE, "staging holds %zu bytes, one slot needs %zu", staging_bytes, slot_bytes);
    int n_slots = (int)(staging_bytes / slot_bytes < (size_t)kMaxOffloadLayers ? staging_bytes / slot_bytes : kMaxOffloadLayers);
    if ((int64_t)k > ceil_div(shape->ctx_len, block))
        return fail(ctx, HYLRA_ERR_BAD_ARG, "k = %d exceeds the %s of the cache", k, block == 1 ? "rows" : "blocks");

    DeviceGuard guard(ctx->device);
    if (!ctx->off_ev) {
        ctx->off_ev = new (std::nothrow) hipEvent_t[1 + 2 * kMaxOffloadLayers]();
        if (!ctx->off_ev) return fail(ctx, HYLRA_ERR_HIP, "out of host memory");
        for (int i = 0; i < 1 + 2 * kMaxOffloadLayers; ++i)
            HIP_TRY(ctx, hipEventCreateWithFlags(&ctx->off_ev[i], hipEventDisableTiming));
    }
    hipEvent_t& ev_idx = ctx->off_ev[0];
    hipEvent_t* ev_gathered = ctx->off_ev + 1;                       // per layer
    hipEvent_t* ev_consumed = ctx->off_ev + 1 + kMaxOffloadLayers;   // per slot
    hipStream_t cs = (hipStream_t)compute_stream, xs = (hipStream_t)copy_stream;

    // the compacted cache of a Reuse layer: `rows` rows per (batch, KV head), contiguous,
    // every sequence the same (slots that hold no row are padding entries of its index set)
    hylra_shape compact = *shape;
    compact.ctx_len = rows;
    compact.kv_stride_b = compact.kv_stride_h = compact.kv_stride_n = 0;

    std::vector<int> slot_of(n_layers, -1);
    std::vector<char> slot_used(n_slots, 0);
    int next_slot = 0;
    // enqueue the gather of Reuse layer r into the next slot (after whoever used the slot last)
    auto prefetch = [&](int r) -> hylra_status {
        const int s = next_slot;
        next_slot = (next_slot + 1) % n_slots;
        if (slot_used[s]) HIP_TRY(ctx, hipStreamWaitEvent(xs, ev_consumed[s], 0));
        const Slot sl = slot_at(staging, shape, rows, s);
        hylra_status rc = gather_impl(ctx, shape, pg, K_l[r], V_l[r], idx_buf, block, k, sl.K, sl.V, sl.idx, xs);
        if (rc != HYLRA_OK) return rc;
        HIP_TRY(ctx, hipEventRecord(ev_gathered[r], xs));
        slot_of[r] = s;
        slot_used[s] = 1;
        return HYLRA_OK;
    };

    int run_end = 0, next_fetch = 0;      // the Reuse layers of the current run are [.., run_end); next to prefetch
    for (int l = 0; l < n_layers; ++l) {
        if (policy[l] == HYLRA_FULL) {
            const bool want_idx = l + 1 == n_layers || policy[l + 1] == HYLRA_REUSE ||
                                  (ctx->flags & HYLRA_FLAG_TOPK_EVERY_FULL_LAYER);
            hylra_status rc = full_impl(ctx, shape, pg, q_l[l], K_l[l], V_l[l], block, k, out_l[l], idx_buf, cs, want_idx);
            if (rc != HYLRA_OK) return rc;
            run_end = l + 1;
            while (run_end < n_layers && policy[run_end] == HYLRA_REUSE) ++run_end;
            next_fetch = l + 1;
            if (next_fetch < run_end) {
                // the run's gathers read this layer's index set
                HIP_TRY(ctx, hipEventRecord(ev_idx, cs));
                HIP_TRY(ctx, hipStreamWaitEvent(xs, ev_idx, 0));
                for (int i = 0; i < n_slots && next_fetch < run_end; ++i, ++next_fetch)
                    if ((rc = prefetch(next_fetch)) != HYLRA_OK) return rc;
            }
        } else {
            const int s = slot_of[l];
            const Slot sl = slot_at(staging, shape, rows, s);
            HIP_TRY(ctx, hipStreamWaitEvent(cs, ev_gathered[l], 0));
            hylra_status rc = reuse_impl(ctx, &compact, nullptr, q_l[l], sl.K, sl.V, sl.idx, 1, rows, out_l[l], cs);
            if (rc != HYLRA_OK) return rc;
            HIP_TRY(ctx, hipEventRecord(ev_consumed[s], cs));
            if (next_fetch < run_end) {
                if ((rc = prefetch(next_fetch)) != HYLRA_OK) return rc;
                ++next_fetch;
            }
        }
    }
    return HYLRA_OK;
}
}  // namespace

hylra_status hylra_decode_step_offloaded(hylra_ctx* ctx, const hylra_shape* shape, int32_t n_layers,
                                         const uint8_t* policy, const void* const* q_l, const void* const* K_l,
                                         const void* const* V_l, int32_t k, float* const* out_l, int32_t* idx_buf,
                                         void* staging, size_t staging_bytes, void* compute_stream,
                                         void* copy_stream) {
    return offloaded_impl(ctx, shape, nullptr, n_layers, policy, q_l, K_l, V_l, 1, k, out_l, idx_buf, staging,
                          staging_bytes, compute_stream, copy_stream);
}

hylra_status hylra_decode_step_offloaded_blocks(hylra_ctx* ctx, const hylra_shape* shape, const hylra_paged* cache,
                                                int32_t n_layers, const uint8_t* policy, const void* const* q_l,
                                                const void* const* K_l, const void* const* V_l, int32_t block,
                                                int32_t kb, float* const* out_l, int32_t* bidx_buf, void* staging,
                                                size_t staging_bytes, void* compute_stream, void* copy_stream) {
    return offloaded_impl(ctx, shape, cache, n_layers, policy, q_l, K_l, V_l, block, kb, out_l, bidx_buf, staging,
                          staging_bytes, compute_stream, copy_stream);
}

hylra_status hylra_overlap_counts(hylra_ctx* ctx, int32_t n_layers, const int32_t* const* idx_l, int32_t batch,
                                  int32_t n_kv_heads, int32_t k, int32_t ctx_len, int64_t* counts,
                                  void* hip_stream) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    if (n_layers < 1 || !idx_l || !counts || ((uintptr_t)counts & 7))
        return fail(ctx, HYLRA_ERR_BAD_ARG, "n_layers < 1, a NULL argument, or counts not 8-byte aligned");
    if (n_layers > kMaxProfileLayers) return fail(ctx, HYLRA_ERR_UNSUPPORTED, "at most %d layers", kMaxProfileLayers);
    if (batch < 1 || n_kv_heads < 1 || k < 1 || ctx_len < 1 || batch > 65535 || n_kv_heads > 65535)
        return fail(ctx, HYLRA_ERR_BAD_ARG, "batch, n_kv_heads (each 1..65535), k and ctx_len must be >= 1");
    if (ctx_len > (1 << 19)) return fail(ctx, HYLRA_ERR_UNSUPPORTED, "ctx_len must be <= %d here", 1 << 19);
    OverlapParams op{};
    for (int l = 0; l < n_layers; ++l) {
        if (!idx_l[l] || ((uintptr_t)idx_l[l] & 3))
            return fail(ctx, HYLRA_ERR_BAD_ARG, "idx_l[%d] must be a 4-byte aligned device pointer", l);
        op.idx[l] = idx_l[l];
    }
    op.L = n_layers, op.Hkv = n_kv_heads, op.k = k, op.N = ctx_len;
    op.counts = reinterpret_cast<unsigned long long*>(counts);
    DeviceGuard guard(ctx->device);
    HIP_TRY(ctx, launch_overlap_counts(op, batch, (hipStream_t)hip_stream));
    return HYLRA_OK;
}

hylra_status hylra_similarity_matrix(int32_t n_layers, const int64_t* counts, double* M) {
    if (n_layers < 1 || !counts || !M) return HYLRA_ERR_BAD_ARG;
    similarity_from_counts(n_layers, counts, M);
    return HYLRA_OK;
}

hylra_status hylra_policy_search(hylra_ctx* ctx, int32_t n_layers, const double* M, double theta, uint8_t* policy,
                                 int32_t* n_full, double* sum_sim) {
    if (n_layers < 1 || !M || !policy) return fail(ctx, HYLRA_ERR_BAD_ARG, "n_layers < 1 or a NULL argument");
    if (!(theta == theta)) return fail(ctx, HYLRA_ERR_BAD_ARG, "theta is not a number");
    const int c = policy_search_host(n_layers, M, theta, policy, sum_sim);
    if (n_full) *n_full = c;
    return HYLRA_OK;
}

hylra_status hylra_profile_enable(hylra_ctx* ctx, int32_t on) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    DeviceGuard guard(ctx->device);
    if (on && !ctx->prof_ev) {
        ctx->prof_ev = new (std::nothrow) hipEvent_t[2 * HYLRA_PROFILE_MAX_EVENTS]();
        if (!ctx->prof_ev) return fail(ctx, HYLRA_ERR_HIP, "out of host memory");
        for (int i = 0; i < 2 * HYLRA_PROFILE_MAX_EVENTS; ++i) HIP_TRY(ctx, hipEventCreate(&ctx->prof_ev[i]));
    }
    if (!on) HIP_TRY(ctx, close_bracket(ctx));
    ctx->prof_on = on != 0;
    return HYLRA_OK;
}

hylra_status hylra_profile_reset(hylra_ctx* ctx) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    {
        DeviceGuard guard(ctx->device);
        HIP_TRY(ctx, close_bracket(ctx));
    }
    ctx->prof_n = 0;
    return HYLRA_OK;
}

hylra_status hylra_profile_read(hylra_ctx* ctx, int32_t kernel_class, int32_t* n_launches, double* total_ms) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    if (kernel_class < 0 || kernel_class >= HYLRA_PROFILE_CLASSES || !n_launches || !total_ms)
        return fail(ctx, HYLRA_ERR_BAD_ARG, "kernel_class outside 0..%d or NULL output", HYLRA_PROFILE_CLASSES - 1);
    DeviceGuard guard(ctx->device);
    HIP_TRY(ctx, close_bracket(ctx));
    int n = 0;
    double ms = 0.0;
    for (int i = 0; i < ctx->prof_n; ++i) {
        if (ctx->prof_cls[i] != kernel_class) continue;
        HIP_TRY(ctx, hipEventSynchronize(ctx->prof_ev[2 * i + 1]));
        float t = 0.f;
        HIP_TRY(ctx, hipEventElapsedTime(&t, ctx->prof_ev[2 * i], ctx->prof_ev[2 * i + 1]));
        ms += t;
        n += ctx->prof_cnt[i];
    }
    *n_launches = n;
    *total_ms = ms;
    return HYLRA_OK;
}

hylra_status hylra_probe_copy(hylra_ctx* ctx, void* dst, const void* src, size_t bytes, void* hip_stream) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    if (!dst || !src || bytes == 0 || bytes % 16 || (((uintptr_t)dst | (uintptr_t)src) & 15))
        return fail(ctx, HYLRA_ERR_BAD_ARG, "probe_copy needs 16-byte aligned pointers and a multiple of 16 bytes");
    hipStream_t st = (hipStream_t)hip_stream;
    DeviceGuard guard(ctx->device);
    HIP_TRY(ctx, launch_timed(ctx, 4, st, [&] { return launch_probe_copy(dst, src, bytes, st); }));
    return HYLRA_OK;
}

hylra_status hylra_probe_gather(hylra_ctx* ctx, const hylra_shape* shape, const void* K, const void* V,
                                const int32_t* idx, int32_t k, void* sink, void* hip_stream) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    int G = 0;
    Strides sd{};
    float scale = 0.f;
    hylra_status rc = check_shape(ctx, shape, G, sd, scale);
    if (rc != HYLRA_OK) return rc;
    if (!K || !V || !idx || !sink || k < 1 || (((uintptr_t)K | (uintptr_t)V | (uintptr_t)sink) & 15) || ((uintptr_t)idx & 3))
        return fail(ctx, HYLRA_ERR_BAD_ARG, "probe_gather needs 16-byte aligned K, V, sink, a 4-byte aligned idx and k >= 1");
    GatherParams gp{};
    gp.K = (const uint16_t*)K, gp.V = (const uint16_t*)V;
    gp.sb = sd.b, gp.sh = sd.h, gp.sn = sd.n;
    gp.Hkv = shape->n_kv_heads, gp.D = shape->head_dim, gp.N = shape->ctx_len, gp.k = k;
    gp.idx = idx;
    hipStream_t st = (hipStream_t)hip_stream;
    DeviceGuard guard(ctx->device);
    HIP_TRY(ctx, launch_timed(ctx, 4, st, [&] { return launch_probe_gather(gp, shape->batch, ctx->n_cus, sink, st); }));
    return HYLRA_OK;
}

hylra_status hylra_probe_read(hylra_ctx* ctx, const void* src, size_t bytes, void* sink, void* hip_stream) {
    if (!ctx) return HYLRA_ERR_BAD_ARG;
    if (!sink || !src || bytes == 0 || bytes % 16 || (((uintptr_t)sink | (uintptr_t)src) & 15))
        return fail(ctx, HYLRA_ERR_BAD_ARG, "probe_read needs 16-byte aligned pointers and a multiple of 16 bytes");
    hipStream_t st = (hipStream_t)hip_stream;
    DeviceGuard guard(ctx->device);
    HIP_TRY(ctx, launch_timed(ctx, 4, st, [&] { return launch_probe_read(src, bytes, sink, st); }));
    return HYLRA_OK;
}

}  // extern "C"
