// Small helpers shared by the matrix-core kernels: operand vector types, a DPP move, and the
// byte permutes that bring bf16 pairs into MFMA operand order.
#pragma once
#include "common.h"

namespace tidal {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

__device__ __forceinline__ s16x4 pack_pairs(uint32_t a1, uint32_t a0, uint32_t b1, uint32_t b0, uint32_t sel) {
    const uint32_t d0 = __builtin_amdgcn_perm(a1, a0, sel), d1 = __builtin_amdgcn_perm(b1, b0, sel);
    return __builtin_bit_cast(s16x4, make_uint2(d0, d1));
}

// Reductions over the four 16-lane rows of a wave, lane by lane within the rows (lanes l, l ^ 16,
// l ^ 32, l ^ 48 all end with the same value): v_permlane32_swap pairs the wave's halves and
// v_permlane16_swap the odd with the even rows, in the vector ALU instead of the LDS crossbar.
__device__ __forceinline__ float cross_rows_max(float v) {
    const auto h = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(h[0]), __uint_as_float(h[1]));
    const auto q = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(q[0]), __uint_as_float(q[1]));
}
__device__ __forceinline__ float cross_rows_sum(float v) {
    const auto h = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(h[0]) + __uint_as_float(h[1]);
    const auto q = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}

constexpr uint32_t kLowHalves = 0x05040100u;   // (x1.lo16 << 16) | x0.lo16
constexpr uint32_t kHighHalves = 0x07060302u;  // (x1.hi16 << 16) | x0.hi16

}  // namespace
}  // namespace tidal
