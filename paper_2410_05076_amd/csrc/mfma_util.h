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

constexpr uint32_t kLowHalves = 0x05040100u;   // (x1.lo16 << 16) | x0.lo16
constexpr uint32_t kHighHalves = 0x07060302u;  // (x1.hi16 << 16) | x0.hi16

}  // namespace
}  // namespace tidal
