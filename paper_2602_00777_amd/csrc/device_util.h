// Small device-side helpers for gfx950 (wave64): bf16 unpacking, the packed bf16 dot
// product, DPP reductions inside a 16-lane row, and the order-preserving float key.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define DEVI __device__ __forceinline__

namespace hylra {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// c + a.lo*b.lo + a.hi*b.hi with a, b holding two bf16 each (v_dot2c_f32_bf16).
// bf16 products are exact in fp32, the accumulation is fp32.
DEVI float dot2_bf16(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a),
                                           __builtin_bit_cast(bf16x2_t, b), c, false);
}

DEVI float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
DEVI float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

DEVI float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int CTRL>
DEVI float dpp_move(float v) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// Sum over aligned groups of LANES lanes (4, 8 or 16); every lane ends with the total.
// quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror, row_mirror.
template <int LANES>
DEVI float group_sum(float v) {
    static_assert(LANES == 4 || LANES == 8 || LANES == 16, "group of 4, 8 or 16 lanes");
    v += dpp_move<0xB1>(v);
    v += dpp_move<0x4E>(v);
    if (LANES >= 8) v += dpp_move<0x141>(v);
    if (LANES >= 16) v += dpp_move<0x140>(v);
    return v;
}

// Unsigned key with the same order as the float (negative zero below positive zero).
DEVI uint32_t ordered_key(float f) {
    uint32_t u = __float_as_uint(f);
    return u ^ ((u >> 31) ? 0xffffffffu : 0x80000000u);
}

// Device-scope relaxed accesses: performed at the point where all compute units of the GPU
// agree (each group of compute units has its own L2), so a value written by one workgroup
// can be read by another during the same launch once the writer's store has completed.
DEVI void coherent_store(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
DEVI float coherent_load(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Wait until every vector memory operation this wave has issued is complete.
DEVI void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Phase timestamps for kernel tuning; compiled in only with -DHYLRA_TRACE (never in the
// product build).  Slot s of workgroup w lands in trace[w * 16 + s] (100 MHz wall clock).
#ifdef HYLRA_TRACE
extern __device__ long long* g_trace;
#define HYLRA_TS(slot)                                                                       \
    do {                                                                                     \
        if (threadIdx.x == 0 && g_trace)                                                     \
            g_trace[((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) * 16 +  \
                    (slot)] = wall_clock64();                                                \
    } while (0)
#else
#define HYLRA_TS(slot) do { } while (0)
#endif

constexpr float NEG_BIG = -1.0e30f;   // "minus infinity" that stays finite under subtraction
constexpr float LOG2E = 1.4426950408889634f;

}  // namespace hylra
