// Small device-side helpers for gfx950 (wave64): bf16 unpacking, the packed bf16 dot
// product, DPP reductions inside a 16-lane row, and the order-preserving float key.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "launch.h"
#include "trace.h"

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

// Register exchanges between the four 16-lane rows of a wave (gfx950 VALU, no LDS traffic).
// swap_rows16(a, b): rows 1 and 3 of a trade places with rows 0 and 2 of b.
// swap_rows32(a, b): rows 2 and 3 of a trade places with rows 0 and 1 of b.
// With a == b on entry, a and b leave holding the two partners of an xor-16 (xor-32) lane
// exchange; with different values, a + b afterwards is a's pair sum on the lower partner
// rows and b's on the upper ones, i.e. one step of a halving butterfly.
DEVI void swap_rows16(float& a, float& b) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    a = __uint_as_float(r[0]);
    b = __uint_as_float(r[1]);
}
DEVI void swap_rows32(float& a, float& b) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    a = __uint_as_float(r[0]);
    b = __uint_as_float(r[1]);
}

// Maximum / minimum over the lanes that share (lane % LANES) in a wave, LANES in {1, 4, 8, 16}
// (LANES = 1: over the whole wave); every lane ends with the result.  row_ror:n rotates within
// a 16-lane row, so rotations by 8 and 4 (and 2, 1) reach every lane of a row.
template <int LANES, bool MAX>
DEVI float strided_minmax(float v) {
    auto op = [](float a, float b) { return MAX ? fmaxf(a, b) : fminf(a, b); };
    if (LANES <= 8) v = op(v, dpp_move<0x128>(v));
    if (LANES <= 4) v = op(v, dpp_move<0x124>(v));
    if (LANES <= 2) v = op(v, dpp_move<0x122>(v));
    if (LANES <= 1) v = op(v, dpp_move<0x121>(v));
    float a = v, b = v;
    swap_rows16(a, b);
    v = op(a, b);
    a = v, b = v;
    swap_rows32(a, b);
    return op(a, b);
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
// Wait until every vector memory operation this wave has issued is complete: s_waitcnt with
// vmcnt = 0 and the other counters left alone.  The immediate's fields on gfx9: vmcnt low four
// bits in [3:0] and its two high bits in [15:14]; expcnt in [6:4] (7 = do not wait); lgkmcnt in
// [11:8] (15 = do not wait).
constexpr int kWaitcntVm0 = (0 << 0) | (0 << 14) | (7 << 4) | (15 << 8);
static_assert(kWaitcntVm0 == 0x0F70, "vmcnt(0), expcnt and lgkmcnt at their no-wait maxima");
DEVI void wait_vmem() { __builtin_amdgcn_s_waitcnt(kWaitcntVm0); }

// Rows of sequence b (see RowMap): clamped to 0..N.
template <class MAP>
DEVI int seq_rows(const MAP& m, int b, int N) {
    return m.seq_lens ? min(max(m.seq_lens[b], 0), N) : N;
}
DEVI int seq_rows(const int32_t* seq_lens, int b, int N) {
    return seq_lens ? min(max(seq_lens[b], 0), N) : N;
}
// The partials of a (batch, KV head) pair: S of them per head, head h's at entries
// base + h * S .. base + (h + 1) * S - 1 of the partial arrays; their score ranges at entries
// first .. first + S - 1 of the range array.
struct PartView {
    int64_t first;
    int S;
};
DEVI PartView part_view(const int2* pair_map, int64_t pair, int n_splits) {
    PartView v;
    v.first = pair * n_splits, v.S = n_splits;
    if (pair_map) {
        const int2 m = pair_map[pair];
        v.first = m.x, v.S = m.y;
    }
    return v;
}

// Units of `block` rows (the last one may be short) that sequence b has, out of at most n_units.
DEVI int seq_units(const int32_t* seq_lens, int b, int n_units, int block) {
    if (!seq_lens) return n_units;
    const int len = seq_lens[b];
    return len <= 0 ? 0 : min((len - 1) / block + 1, n_units);
}
// Element offset of row `row` of sequence b from the (batch-independent) base of a paged pool;
// tbl points at the sequence's row of the page table (in memory or staged in LDS).
template <class MAP>
DEVI int64_t paged_row_offset(const MAP& m, const int32_t* tbl, int row, int64_t sn) {
    return (int64_t)tbl[row >> m.page_shift] * m.stride_page + (int64_t)(row & ((1 << m.page_shift) - 1)) * sn;
}

constexpr float NEG_BIG = -1.0e30f;   // "minus infinity" that stays finite under subtraction
constexpr float LOG2E = 1.4426950408889634f;

}  // namespace hylra
