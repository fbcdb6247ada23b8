// Phase timestamps for kernel tuning.  Everything here is compiled in only with -DHYLRA_TRACE
// (a tuning build; the product build defines nothing and HYLRA_TS expands to nothing).
// Slot s of workgroup w lands in trace[w * 16 + s] (100 MHz wall clock).  The translation unit
// that defines HYLRA_TRACE_OWNER before including this header holds the buffer pointer and the
// entry point that sets it.
#pragma once
#ifdef HYLRA_TRACE
#include <hip/hip_runtime.h>
namespace hylra {
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
#define HYLRA_TS(slot)                                                                       \
    do {                                                                                     \
        if (threadIdx.x == 0 && hylra::g_trace)                                              \
            hylra::g_trace[((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * 16 + \
                           (slot)] = wall_clock64();                                         \
    } while (0)
#else
#define HYLRA_TS(slot) do { } while (0)
#endif
