// Device helpers shared by the bf16 MFMA attention kernels (gfx950, wave64).
//
// MFMA used: v_mfma_f32_32x32x16_bf16.  Operand layout, lane l = 32*hl + m (m = l % 32):
//   A (32 x 16): lane holds row m,    k = 8*hl .. 8*hl+7   (8 bf16 = 16 bytes)
//   B (16 x 32): lane holds column m, k = 8*hl .. 8*hl+7
//   C (32 x 32): lane holds column m, register c = 4*g + r  <->  row 8*g + 4*hl + r
// Every kernel here computes "transposed" score tiles (rows = keys or queries of the streamed
// tile, columns = the rows the wavefront owns), so each lane owns one of the wavefront's rows
// and per-row softmax statistics are per-lane scalars.
#pragma once
#include <hip/hip_runtime.h>

namespace mate {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));

constexpr int kD = 64;             // head size
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ inline f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ inline f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int i = 0; i < 16; ++i) z[i] = 0.f;
  return z;
}

// Registers c0 .. c0+7 of a C tile, rounded to bf16 (nearest even), as an MFMA operand.
__device__ inline bf16x8 pack8(const f32x16& x, int c0) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (__bf16)x[c0 + e];
  return r;
}

// max / sum of a per-row value across the two lane halves that share the row (lanes l, l ^ 32):
// v_permlane32_swap exchanges the upper half of its first operand with the lower half of the
// second, so after swapping (x, x) every lane holds both halves' values.
__device__ inline float half_max(float x) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float half_sum(float x) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Sum of the eight bf16 values of an operand, added to acc (v_dot2 against ones): the row sum
// of exactly the rounded probabilities that go into the second contraction.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ inline float sum8(bf16x8 p, float acc) {
  const bf16x2 one = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const bf16x2 pr = {p[2 * e], p[2 * e + 1]};
    acc = __builtin_amdgcn_fdot2_f32_bf16(pr, one, acc, false);
  }
  return acc;
}

__device__ inline bf16x8 as_bf16x8(uint4 v) {
  union { uint4 u; bf16x8 b; } x;
  x.u = v;
  return x.b;
}

__device__ inline unsigned short f32_to_bf16_bits(float x) {
  __bf16 h = (__bf16)x;
  return __builtin_bit_cast(unsigned short, h);
}

}  // namespace mate
