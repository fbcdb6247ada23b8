// Offline profiling step that produces the layer policy (paper: "Inter-Layer Similarity",
// Eq. 2; "Offline Optimal Policy via Dynamic Programming", Algorithm 1).
//
//   overlap counts   for layers i <= j: the sum over all (batch, KV head) sets of |S_i ∩ S_j|,
//                    S_l being the index set a Full layer produced at layer l.  One workgroup
//                    per (layer j, KV head, batch) marks S_j in a bitmap of ctx_len bits in
//                    LDS and tests the entries of S_0 .. S_j against it.  Integer work, exact.
//   policy search    host code: the path search of Algorithm 1 over the similarity matrix
//                    M[i][j] = counts[i][j] / counts[j][j].
#include <vector>

#include "device_util.h"
#include "launch.h"

namespace hylra {

__global__ __launch_bounds__(256) void overlap_zero_kernel(unsigned long long* counts, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) counts[i] = 0;
}

__global__ __launch_bounds__(256) void overlap_counts_kernel(OverlapParams p) {
    extern __shared__ uint32_t s_bits[];            // ceil(N / 32) words
    __shared__ int s_part[4];
    const int j = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t set = ((int64_t)b * p.Hkv + g) * p.k;
    const int words = (p.N + 31) >> 5;

    for (int w = tid; w < words; w += 256) s_bits[w] = 0;
    __syncthreads();
    const int32_t* __restrict__ sj = p.idx[j] + set;
    for (int t = tid; t < p.k; t += 256) {
        const int v = sj[t];
        if ((unsigned)v < (unsigned)p.N) atomicOr(&s_bits[v >> 5], 1u << (v & 31));
    }
    __syncthreads();
    for (int i = 0; i <= j; ++i) {
        const int32_t* __restrict__ si = p.idx[i] + set;
        int c = 0;
        for (int t = tid; t < p.k; t += 256) {
            const int v = si[t];
            if ((unsigned)v < (unsigned)p.N) c += (s_bits[v >> 5] >> (v & 31)) & 1u;
        }
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) c += __shfl_xor(c, m, 64);
        if (lane == 0) s_part[wave] = c;
        __syncthreads();
        if (tid == 0) {
            const int total = s_part[0] + s_part[1] + s_part[2] + s_part[3];
            if (total) atomicAdd(p.counts + (int64_t)i * p.L + j, (unsigned long long)total);
        }
        __syncthreads();
    }
}

hipError_t launch_overlap_counts(const OverlapParams& p, int B, hipStream_t st) {
    const int n = p.L * p.L;
    hipLaunchKernelGGL(overlap_zero_kernel, dim3((n + 255) / 256), dim3(256), 0, st, p.counts, n);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t lds = (size_t)((p.N + 31) >> 5) * sizeof(uint32_t);
    hipLaunchKernelGGL(overlap_counts_kernel, dim3(p.L, p.Hkv, B), dim3(256), lds, st, p);
    return hipGetLastError();
}

}  // namespace hylra
