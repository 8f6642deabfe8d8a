// Device helpers shared by the bf16 matrix-core attention kernels (gfx950 only).
//
// Matrix instruction used: v_mfma_f32_32x32x16_bf16, D[32x32] += A[32x16] * B[16x32], one wave.
// Register layout (lane l, c = l % 32, g = l / 32):
//   A: lane holds row c,    k = 8g .. 8g+7   (8 consecutive bf16 = one 16-byte register group)
//   B: lane holds column c, k = 8g .. 8g+7
//   D: lane holds column c, rows 8*(v/4) + 4g + (v%4) for accumulator register v = 0..15
// The k index is summed away, so any permutation of k may be used as long as A and B agree; the
// kernels use that to feed an accumulator tile straight back as the B operand of the next product.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mb {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 x) { return __builtin_bit_cast(bf16x8, x); }

// Two floats -> two bf16 (round to nearest even) packed in one 32-bit register, lo in bits 0..15.
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  bf16x2 r;
  r[0] = (__bf16)lo;
  r[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, r);
}

// Eight accumulator floats -> one bf16x8 operand.
__device__ __forceinline__ bf16x8 pack8(float a0, float a1, float a2, float a3, float a4, float a5, float a6,
                                        float a7) {
  u32x4 r;
  r[0] = pack_bf16(a0, a1);
  r[1] = pack_bf16(a2, a3);
  r[2] = pack_bf16(a4, a5);
  r[3] = pack_bf16(a6, a7);
  return as_bf16x8(r);
}

// Value of x held by the partner lane (l ^ 32), via v_permlane32_swap.
__device__ __forceinline__ float other_half(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);  // r[0]: lower half's x, r[1]: upper half's
  return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}
__device__ __forceinline__ float max_both_halves(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_both_halves(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// 16 bytes (8 bf16) from LDS.
__device__ __forceinline__ bf16x8 lds_read8(const uint16_t* p) {
  return as_bf16x8(*reinterpret_cast<const u32x4*>(p));
}

// Transposing LDS read (ds_read_b64_tr_b16).  Within each group of 16 lanes, lane i passes the address
// of 4 consecutive bf16: row (i / 4) of a 4-row patch, columns 4*(i % 4) .. +3 of a 16-column window.
// Lane i receives column i of the patch: the 4 values of rows 0..3.
__device__ __forceinline__ s16x4 lds_read_tr4(const uint16_t* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) s16x4*)(const_cast<uint16_t*>(p)));
}
__device__ __forceinline__ bf16x8 join_tr(s16x4 lo, s16x4 hi) {
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  s16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, r);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

}  // namespace mb
