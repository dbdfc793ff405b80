// Small device-side helpers for gfx950 shared by the kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "loong.h"

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

// ---- 16-bit storage types.  The kernels keep operand fragments as eight 16-bit lanes in a
// bf16x8_t whatever the element type is; the element class says how the matrix instruction
// reads them and how fp32 values are rounded into them (nearest even for both).
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));

struct Bf16 {
  static constexpr int code = LOONG_BF16;
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) { return pack_bf16x2(lo, hi); }
  static __device__ __forceinline__ float lo(uint32_t w) { return bf16_lo(w); }
  static __device__ __forceinline__ float hi(uint32_t w) { return bf16_hi(w); }
  static __device__ __forceinline__ floatx16_t mfma(bf16x8_t a, bf16x8_t b, floatx16_t c) { return mfma32(a, b, c); }
};

struct Fp16 {
  static constexpr int code = LOONG_FP16;
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    floatx2_t f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, f16x2_t));
  }
  static __device__ __forceinline__ float lo(uint32_t w) { return (float)__builtin_bit_cast(f16x2_t, w)[0]; }
  static __device__ __forceinline__ float hi(uint32_t w) { return (float)__builtin_bit_cast(f16x2_t, w)[1]; }
  static __device__ __forceinline__ floatx16_t mfma(bf16x8_t a, bf16x8_t b, floatx16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
  }
};

// An operand fragment with every element multiplied by c (rounded to the storage type again).
template <class E>
__device__ __forceinline__ bf16x8_t scaled_fragment(bf16x8_t f, float c) {
  const uint4 w = __builtin_bit_cast(uint4, f);
  return as_bf16x8(make_uint4(E::pack2(E::lo(w.x) * c, E::hi(w.x) * c), E::pack2(E::lo(w.y) * c, E::hi(w.y) * c),
                              E::pack2(E::lo(w.z) * c, E::hi(w.z) * c), E::pack2(E::lo(w.w) * c, E::hi(w.w) * c)));
}

// Row index inside a 32x32 accumulator block held in register v of a lane of half hh.
__device__ __forceinline__ constexpr int acc_row(int v, int hh) { return 8 * (v >> 2) + 4 * hh + (v & 3); }

// Maximum / sum of a value with that of the lane 32 places away (wave64), on the vector ALU
// (v_permlane32_swap: no LDS round trip, and no wait that would also cover the LDS reads in
// flight).  After the swap one result holds lanes 0-31 of x in both halves, the other lanes
// 32-63 in both halves; the operations are symmetric, so no selection by half is needed.
typedef unsigned uintx2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float max_with_other_half(float x) {
  const uintx2_t r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_with_other_half(float x) {
  const uintx2_t r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// The value of the lane one (two) places away inside each group of four lanes.
__device__ __forceinline__ float quad_swap1(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, x), 0xB1, 0xf, 0xf, false));  // quad_perm [1,0,3,2]
}
__device__ __forceinline__ float quad_swap2(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, x), 0x4E, 0xf, 0xf, false));  // quad_perm [2,3,0,1]
}

// ---- global memory -> LDS without registers -------------------------------------------------
// 16 (or 4) bytes per lane from global memory straight into LDS: lane l's data lands at
// lds_addr + 16 l (4 l), lds_addr uniform over the wave.  Written as assembly so that the
// compiler does not tie every later LDS read to the completion of all loads in flight; the
// kernels wait for the data they need with wait_vmcnt.  The statements clobber "memory": they
// write LDS behind the compiler's back, so it must not move LDS accesses across them.
__device__ __forceinline__ void load_to_lds_16(const void* gptr, uint32_t lds_addr) {
  const uint32_t uniform_addr = __builtin_amdgcn_readfirstlane(lds_addr);
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(uniform_addr) : "m0", "memory");
}
__device__ __forceinline__ void load_to_lds_4(const void* gptr, uint32_t lds_addr) {
  const uint32_t uniform_addr = __builtin_amdgcn_readfirstlane(lds_addr);
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dword %0, off" ::"v"(gptr), "s"(uniform_addr) : "m0", "memory");
}

// The same with the address split into a wave-uniform 64-bit base (scalar registers) and a
// 32-bit per-lane byte offset: no 64-bit vector arithmetic per load.
__device__ __forceinline__ void load_to_lds_16(const void* uniform_base, uint32_t lane_off, uint32_t lds_addr) {
  const uint64_t a = reinterpret_cast<uint64_t>(uniform_base);
  // (the builtin returns a signed int: convert each half back to unsigned before widening)
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)a);
  const uint64_t base = ((uint64_t)hi << 32) | (uint64_t)lo;
  const uint32_t uniform_addr = __builtin_amdgcn_readfirstlane(lds_addr);
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(base), "s"(uniform_addr) : "m0", "memory");
}

// s_waitcnt vmcnt(n) with the other counters left alone (gfx9 encoding)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// Transposing LDS read: in every group of 16 lanes, lane i points at 8 bytes: row i / 4 of a
// run of four rows, columns 4 (i % 4) .. +3 of a 16-column strip of 16-bit elements; it
// receives the four rows' values of column i of the strip.
typedef short v4i16_t __attribute__((ext_vector_type(4)));
typedef short v8i16_t __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) v4i16_t lds_v4i16_t;
__device__ __forceinline__ bf16x8_t read_tr_pair(const unsigned char* lo_run, const unsigned char* hi_run) {
  const v4i16_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_t*)lo_run);
  const v4i16_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16_t*)hi_run);
  return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// XOR applied to the 16-byte piece index of row `row` of an unpadded row-major 16-bit tile in
// LDS with D columns, chosen so that both access patterns of the kernels are free of bank
// conflicts.  The LDS serves 256 bytes (64 banks) per clock: a 16-byte read takes 16 lanes per
// clock, which here read the same piece of 16 consecutive rows, so the XOR must differ for
// all of them; an 8-byte transposing read takes 32 lanes per clock, which here cover four
// consecutive rows x four adjacent pieces, so the four rows' XORs must differ in the bits
// above those two (the SQ_LDS_BANK_CONFLICT counter reads zero with this choice; with the
// four rows only two pieces apart it read half of the transposing reads' cycles).
template <int D>
__device__ __forceinline__ constexpr int tile_swizzle(int row) {
  if (D == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
  const int m = (row >> 1) & 7;  // D == 64: two rows per 256 bytes
  return ((m & 1) << 2) | ((m >> 1) & 3);
}

// f(integral_constant<int, I>) for I = First .. Last - 1, unrolled by instantiation (does not
// depend on the loop unroller's size limits)
template <int First, int Last, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (First < Last) {
    f(std::integral_constant<int, First>{});
    static_for<First + 1, Last>(f);
  }
}

}  // namespace loong
