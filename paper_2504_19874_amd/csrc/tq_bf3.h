// Exact splitting of fp32 values into bf16 pieces, shared by the kernels that run fp32 contractions on the
// bf16 matrix cores (tq_score_bf3.hip, tq_d128_bf3.hip): x = x1 + x2 + x3 with 8 significand bits each, so a
// product of two pieces is exact in fp32 and the six products of combined weight >= 2^-16 reproduce an fp32
// product to 2^-24.
#pragma once
#include "tq_internal.h"

namespace tq {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t bf16_bits(float x) {  // round to nearest even
  const __bf16 h = (__bf16)x;
  return (uint32_t) * reinterpret_cast<const unsigned short*>(&h);
}

// x -> (x1, x2, x3), three bf16 values with x1 + x2 + x3 == x
__device__ __forceinline__ void split3(float x, uint32_t& p1, uint32_t& p2, uint32_t& p3) {
  p1 = bf16_bits(x);
  const float r1 = x - __uint_as_float(p1 << 16);
  p2 = bf16_bits(r1);
  const float r2 = r1 - __uint_as_float(p2 << 16);
  p3 = bf16_bits(r2);
}

// the same for two values at once: word k holds piece k of x[0] (low half) and of x[1] (high half); one
// packed conversion per piece
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t bf16_pair(f32x2 x) {
  const bf16x2 h = __builtin_convertvector(x, bf16x2);
  return *reinterpret_cast<const uint32_t*>(&h);
}
__device__ __forceinline__ void split3_pair(f32x2 x, uint32_t& w1, uint32_t& w2, uint32_t& w3) {
  w1 = bf16_pair(x);
  const f32x2 r1 = {x[0] - __uint_as_float(w1 << 16), x[1] - __uint_as_float(w1 & 0xffff0000u)};
  w2 = bf16_pair(r1);
  const f32x2 r2 = {r1[0] - __uint_as_float(w2 << 16), r1[1] - __uint_as_float(w2 & 0xffff0000u)};
  w3 = bf16_pair(r2);
}

// the two leading pieces only: x1 + x2 == x up to 2^-17 |x|
__device__ __forceinline__ void split2_pair(f32x2 x, uint32_t& w1, uint32_t& w2) {
  w1 = bf16_pair(x);
  const f32x2 r1 = {x[0] - __uint_as_float(w1 << 16), x[1] - __uint_as_float(w1 & 0xffff0000u)};
  w2 = bf16_pair(r1);
}

}  // namespace tq
