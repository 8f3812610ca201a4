// Device-side helpers shared by the gfx950 kernels: vector types, MFMA
// wrappers, cross-lane exchange, bf16 packing.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sa_kernels.h"

namespace sa {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;  // finite "minus infinity" for running maxima

// D(32x32) += A(32x16) * B(16x32), bf16 in, fp32 accumulate.
// Lane l supplies A[l%32][8*(l/32) .. +7] and B[8*(l/32) .. +7][l%32];
// it receives D[8*(r/4) + 4*(l/32) + r%4][l%32] in element r of the result.
__device__ __forceinline__ f32x16 mfma_32x32x16(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

// value held by the lane 32 positions away (lanes l and l^32 exchange)
__device__ __forceinline__ float swap_half(float x) {
  return __shfl_xor(x, 32, 64);
}

// Lanes l and l^32 each hold x; both receive the pair (x of the lower lane, x of the
// upper lane) through one register swap between the two 32-lane halves: a vector-ALU
// operation, no trip through LDS.
__device__ __forceinline__ void half_pair(float x, float& lo, float& hi) {
  unsigned u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  lo = __uint_as_float(r[0]);
  hi = __uint_as_float(r[1]);
}
__device__ __forceinline__ float half_max(float x) {
  float a, b;
  half_pair(x, a, b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float half_sum(float x) {
  float a, b;
  half_pair(x, a, b);
  return a + b;
}

// round-to-nearest-even fp32 -> bf16 pair packed into one dword (lo = a)
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  typedef __attribute__((ext_vector_type(2))) float f32x2;
  f32x2 f = {a, b};
  bf16x2 h = __builtin_convertvector(f, bf16x2);
  return __builtin_bit_cast(uint32_t, h);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// position inside a 32-row group at which K row `r` is stored in LDS: bits 2
// and 3 of the row index are exchanged so that the score accumulators of one
// lane come out in consecutive-key order (see the flash kernel).
__device__ __forceinline__ int krow_slot(int r) {
  return (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1);
}

}  // namespace sa
