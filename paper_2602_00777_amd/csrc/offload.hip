// Index-guided prefetch (paper: "Bandwidth reduction via index-guided offloading"): the KV
// cache of a tolerant layer lives where the GPU can read it but only slowly (pinned host
// memory across PCIe), and since the layer's index set is known as soon as the preceding
// sensitive layer has run, only the selected rows are fetched, ahead of time, into a compact
// buffer in device memory:
//     K_dst[b, g, t, :] = K_src[b, g, idx[b, g, t], :]      (likewise V)
//     idx_dst[b, g, t]  = t  if idx[b, g, t] names a row, else -1
// after which the Reuse layer is ordinary sparse attention over a cache of k rows with the
// index set idx_dst.  Byte work: bit-exact.
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
    const int32_t* __restrict__ ib = p.idx + pair * p.k;
    const int64_t src_base = (int64_t)b * p.sb + (int64_t)g * p.sh;
    const int pieces = p.D >> 3;
    const int t0 = blockIdx.x * (16 * U);
    int row[U];
    uint4 kv[U], vv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int t = t0 + 16 * u + slot;
        row[u] = t < p.k ? ib[t] : -1;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const bool ok = (unsigned)row[u] < (unsigned)p.N && piece < pieces;
        kv[u] = vv[u] = make_uint4(0, 0, 0, 0);             // padding entries leave zero rows
        if (ok) {
            const int64_t off = src_base + (int64_t)row[u] * p.sn + 8 * piece;
            kv[u] = *reinterpret_cast<const uint4*>(p.K + off);
            vv[u] = *reinterpret_cast<const uint4*>(p.V + off);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int t = t0 + 16 * u + slot;
        if (t >= p.k) continue;
        if (piece < pieces) {
            const int64_t off = (pair * p.k + t) * p.D + 8 * piece;
            *reinterpret_cast<uint4*>(p.K_dst + off) = kv[u];
            *reinterpret_cast<uint4*>(p.V_dst + off) = vv[u];
        }
        if (piece == 0) p.idx_dst[pair * p.k + t] = (unsigned)row[u] < (unsigned)p.N ? t : -1;
    }
}

hipError_t launch_gather_rows(const GatherParams& p, int B, hipStream_t st) {
    constexpr int U = 4;
    const dim3 grid((p.k + 16 * U - 1) / (16 * U), p.Hkv, B);
    hipLaunchKernelGGL(gather_rows_kernel<U>, grid, dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace hylra
