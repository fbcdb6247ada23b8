// Phase timestamps for kernel tuning.  Everything here is compiled in only with -DHYLRA_TRACE
// (a tuning build; the product build defines nothing and the macros expand to nothing).
// Slot s of workgroup w lands in trace[(region * 8192 + w) * 16 + s] (100 MHz wall clock); the
// buffer holds 2 * 8192 * 16 64-bit words.  Region 0: streaming and Reuse kernels (HYLRA_TS);
// region 1: the selection kernels (HYLRA_TS_SEL), which run in the same call as a streaming
// kernel and would otherwise write over its rows.  Workgroups beyond 8192 are not recorded.
// The translation unit that defines HYLRA_TRACE_OWNER before including this header holds the
// buffer pointer and the entry point that sets it.
#pragma once
#ifdef HYLRA_TRACE
#include <hip/hip_runtime.h>
namespace hylra {
constexpr unsigned kTraceRows = 8192;
#ifdef HYLRA_TRACE_OWNER
__device__ long long* g_trace = nullptr;
#else
extern __device__ long long* g_trace;
#endif
}  // namespace hylra
#ifdef HYLRA_TRACE_OWNER
extern "C" int hylra_debug_set_trace(void* device_buffer) {
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(hylra::g_trace), &device_buffer, sizeof(void*));
}
#endif
#define HYLRA_TS_AT(region, slot)                                                                      \
    do {                                                                                               \
        const unsigned hylra_wg_ = (blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;     \
        if (threadIdx.x == 0 && hylra::g_trace && hylra_wg_ < hylra::kTraceRows)                       \
            hylra::g_trace[((region) * hylra::kTraceRows + hylra_wg_) * 16 + (slot)] = wall_clock64(); \
    } while (0)
#define HYLRA_TS(slot) HYLRA_TS_AT(0u, slot)
#define HYLRA_TS_SEL(slot) HYLRA_TS_AT(1u, slot)
#else
#define HYLRA_TS(slot) do { } while (0)
#define HYLRA_TS_SEL(slot) do { } while (0)
#endif
