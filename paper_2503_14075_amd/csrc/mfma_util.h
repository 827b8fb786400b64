// Matrix-core helpers shared by the bf16 kernels (gfx950, wave64).
//
// v_mfma_f32_32x32x16_bf16 operand layouts (lane l, g = l / 32, i = l % 32):
//   A[i][8g + e], B[8g + e][i] for e = 0..7;   D[8*(r/4) + 4g + r%4][i] for r = 0..15.
// A and B hold the same (lane, element) -> reduction-index map, so any
// permutation of the reduction index applied to both operands is free.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tw {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

__device__ __forceinline__ bf16x8 as_bf16x8(const u32x4& v) { return __builtin_bit_cast(bf16x8, v); }

// row of a 32x32 accumulator tile held by register r of lane group g
__device__ __forceinline__ int acc_row(int r, int g) { return 8 * (r >> 2) + 4 * g + (r & 3); }

// v_exp_f32: 2^x at 1 ulp; results below 2^-126 flush to zero, which is what a softmax weight that small is worth
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

}  // namespace tw
