// Index-guided prefetch (paper: "Bandwidth reduction via index-guided offloading": selective
// prefetching of only the critical KV blocks): the KV cache of a tolerant layer lives where the
// GPU can read it but only slowly (pinned host memory across PCIe), and since the layer's index
// set is known as soon as the preceding sensitive layer has run, only the selected rows are
// fetched, ahead of time, into a compact buffer in device memory.  With blocks of `block` rows
// (block = 1: single rows) and kb selected blocks per (batch, KV head), slot p = t * block + r:
//     row(p)            = idx[b, g, t] * block + r
//     K_dst[b, g, p, :] = K_src[b, g, row(p), :]      (likewise V; zeros where row(p) is no row)
//     idx_dst[b, g, p]  = p  if row(p) is a row of sequence b, else -1
// after which the Reuse layer is ordinary token-level sparse attention over a cache of
// kb * block rows with the index set idx_dst.  Byte work: bit-exact.
//
// Also here: the decode-time cache update that precedes Algorithm 2 (its K^cache and V^cache
// hold the current token): the token's key and value rows are written behind the rows each
// sequence already has.
#include "device_util.h"
#include "launch.h"

namespace hylra {

// 16 lanes per row (D = 128: one 16-byte piece per lane; D = 64: lanes 8..15 idle), 16 rows per
// wave-wide instruction of a 256-thread workgroup, U instructions in flight per thread.
template <int U>
__global__ __launch_bounds__(256) void gather_rows_kernel(GatherParams p) {
    const int g = blockIdx.y, b = blockIdx.z;
    const int piece = threadIdx.x & 15, slot = threadIdx.x >> 4;
    const int64_t pair = (int64_t)b * p.Hkv + g;
    const int32_t* __restrict__ ib = p.idx + pair * p.idx_stride;
    const int32_t* __restrict__ tbl = p.map.table ? p.map.table + (int64_t)b * p.map.table_stride : nullptr;
    const int64_t src_base = (tbl ? 0 : (int64_t)b * p.sb) + (int64_t)g * p.sh;
    const int n_rows = seq_rows(p.map, b, p.N);
    const int pieces = p.D >> 3;
    const int t0 = blockIdx.x * (16 * U);
    int row[U];
    uint4 kv[U], vv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int pos = t0 + 16 * u + slot;
        row[u] = -1;
        if (pos < p.k) {
            if (p.block == 1) {
                row[u] = ib[pos];
            } else {
                // pos / block by a multiply-high with ceil(2^32 / block): at most one too large
                int t = (int)__umulhi((uint32_t)pos, p.block_magic);
                if (t * p.block > pos) --t;
                const int c = ib[t];
                if ((unsigned)c < (unsigned)p.n_blocks) row[u] = c * p.block + (pos - t * p.block);
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const bool ok = (unsigned)row[u] < (unsigned)n_rows && piece < pieces;
        kv[u] = vv[u] = make_uint4(0, 0, 0, 0);             // slots that hold no row stay zero
        if (ok) {
            const int64_t off = src_base + (tbl ? paged_row_offset(p.map, tbl, row[u], p.sn) : (int64_t)row[u] * p.sn) + 8 * piece;
            kv[u] = *reinterpret_cast<const uint4*>(p.K + off);
            vv[u] = *reinterpret_cast<const uint4*>(p.V + off);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int pos = t0 + 16 * u + slot;
        if (pos >= p.k) continue;
        if (piece < pieces) {
            const int64_t off = (pair * p.k + pos) * p.D + 8 * piece;
            *reinterpret_cast<uint4*>(p.K_dst + off) = kv[u];
            *reinterpret_cast<uint4*>(p.V_dst + off) = vv[u];
        }
        if (piece == 0) p.idx_dst[pair * p.k + pos] = (unsigned)row[u] < (unsigned)n_rows ? pos : -1;
    }
}

hipError_t launch_gather_rows(const GatherParams& p, int B, hipStream_t st) {
    constexpr int U = 4;
    const dim3 grid((p.k + 16 * U - 1) / (16 * U), p.Hkv, B);
    hipLaunchKernelGGL(gather_rows_kernel<U>, grid, dim3(256), 0, st, p);
    return hipGetLastError();
}

// One workgroup of 64 threads per (KV head, batch): lanes 0..15 copy the key row, lanes 16..31
// the value row (16 bytes each; D = 64 uses half of them).  The row lands at position n_b =
// the sequence's length before the call (clamped to 0 .. N - 1), through the page table if the
// cache is paged.  lens_out[b] = n_b + 1, the length the attention that follows has to use.
__global__ __launch_bounds__(64) void append_rows_kernel(AppendParams p) {
    const int g = blockIdx.x, b = blockIdx.y;
    const int lane = threadIdx.x, piece = lane & 15, which = lane >> 4;
    int n = p.map.seq_lens ? p.map.seq_lens[b] : p.N - 1;
    n = min(max(n, 0), p.N - 1);
    if (g == 0 && lane == 0 && p.lens_out) p.lens_out[b] = n + 1;
    if (which > 1 || piece >= (p.D >> 3)) return;
    const int32_t* __restrict__ tbl = p.map.table ? p.map.table + (int64_t)b * p.map.table_stride : nullptr;
    const int64_t off = (tbl ? paged_row_offset(p.map, tbl, n, p.sn) : (int64_t)b * p.sb + (int64_t)n * p.sn) +
                        (int64_t)g * p.sh + 8 * piece;
    const int64_t src = ((int64_t)b * p.Hkv + g) * p.D + 8 * piece;
    if (which == 0) *reinterpret_cast<uint4*>(p.K + off) = *reinterpret_cast<const uint4*>(p.k_new + src);
    else *reinterpret_cast<uint4*>(p.V + off) = *reinterpret_cast<const uint4*>(p.v_new + src);
}

hipError_t launch_append_rows(const AppendParams& p, int B, hipStream_t st) {
    hipLaunchKernelGGL(append_rows_kernel, dim3(p.Hkv, B), dim3(64), 0, st, p);
    return hipGetLastError();
}

}  // namespace hylra
