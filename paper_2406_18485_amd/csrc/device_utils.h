// Small device-side helpers for gfx950 shared by the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace loong {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Two floats -> two bf16 (round to nearest even) packed in one dword, `lo` in bits 0..15.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  floatx2_t f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ bf16x8_t as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8_t, v); }

// 2^x and log2(x) on the hardware transcendental unit.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// D(32x32, fp32) += A(32x16, bf16) * B(16x32, bf16).  Lane l supplies row (l & 31) of A and
// column (l & 31) of B, eight consecutive contraction indices starting at 8 * (l >> 5);
// it owns column (l & 31) of D, rows 8 * (v / 4) + 4 * (l >> 5) + (v % 4), v = 0..15.
__device__ __forceinline__ floatx16_t mfma32(bf16x8_t a, bf16x8_t b, floatx16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Row index inside a 32x32 accumulator block held in register v of a lane of half hh.
__device__ __forceinline__ constexpr int acc_row(int v, int hh) { return 8 * (v >> 2) + 4 * hh + (v & 3); }

// Value of the lane 32 places away (wave64).
__device__ __forceinline__ float other_half(float x) { return __shfl_xor(x, 32, 64); }

}  // namespace loong
