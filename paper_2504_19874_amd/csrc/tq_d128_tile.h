// The per-tile decision step shared by the d = 128 quantisation kernels.
#pragma once
#include "tq_internal.h"

namespace tq {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Lane l and lane l ^ 32 exchange a register inside the vector unit (no LDS round trip): the pair
// (own value, partner's value) in an order that depends on the half-wave; for commutative merges.
__device__ __forceinline__ uint32_t or_across_halves(uint32_t w) {
  const auto r = __builtin_amdgcn_permlane32_swap(w, w, false, false);
  return r[0] | r[1];
}
__device__ __forceinline__ float add_across_halves(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// nib = 2 nib + bit as ONE add-with-carry whose carry-in is the compare mask itself (written as a select and a
// shift-or otherwise)
__device__ __forceinline__ uint32_t shift_in(uint32_t nib, uint64_t mask) {
  uint64_t carry_out;
  asm("v_addc_co_u32 %0, %1, %2, %2, %3" : "=v"(nib), "=s"(carry_out) : "v"(nib), "s"(mask));
  return nib;
}

// One output tile (32 coordinates x 32 vectors, 16 coordinates per lane) through the decision
// of Alg. 1: nearest centroid, packing, residual (in place).  Bit p of the bucket number is the
// XOR of the compare masks at positions k = 2^p - 1 (mod 2^p); a 4-bit nibble of a plane is
// built by shift-and-add-carry, most significant element first.  Returns the lane's share of
// the squared residual norm; word[p] is the finished plane word (both half-waves merged).
template <int B>
__device__ __forceinline__ float quantise_tile(floatx16& acc, const float inv, const Codebook& cb, const int h,
                                               uint32_t (&word)[4]) {
  float g2 = 0.f;
  uint32_t nib[4][B > 0 ? B : 1];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
#pragma unroll
    for (int pl = 0; pl < (B > 0 ? B : 1); ++pl) nib[k][pl] = 0u;
#pragma unroll
    for (int r = 3; r >= 0; --r) {
      const float y = acc[4 * k + r] * inv;
      float yt = cb.c[0];
      uint64_t bit[B > 0 ? B : 1];  // lane masks, combined on the scalar unit
#pragma unroll
      for (int pl = 0; pl < (B > 0 ? B : 1); ++pl) bit[pl] = 0;
#pragma unroll
      for (int j = 0; j < (1 << B) - 1; ++j) {
        // both table values are read before the select: a read inside one arm of the conditional can be
        // merged by the compiler into ONE indexed load from the table's memory, a round trip per coordinate
        const float tj = cb.t[j], cj = cb.c[j + 1];
        const bool ge = y >= tj;
        yt = ge ? cj : yt;
        const uint64_t gem = __builtin_amdgcn_ballot_w64(ge);
#pragma unroll
        for (int pl = 0; pl < B; ++pl)
          if ((j & ((1 << pl) - 1)) == (1 << pl) - 1) bit[pl] ^= gem;
      }
      float e = y - yt;
      asm volatile("" : "+v"(e));  // keep the residual here: sunk later it would need the masks again
      g2 = fmaf(e, e, g2);
      acc[4 * k + r] = e;
#pragma unroll
      for (int pl = 0; pl < B; ++pl) nib[k][pl] = shift_in(nib[k][pl], bit[pl]);
    }
  }
#pragma unroll
  for (int pl = 0; pl < B; ++pl) {
    const uint32_t w = (nib[0][pl] | (nib[1][pl] << 8) | (nib[2][pl] << 16) | (nib[3][pl] << 24)) << (4 * h);
    word[pl] = or_across_halves(w);
  }
  return g2;
}

// The same for a codebook that is symmetric about zero (c[i] = -c[K-1-i], t[j] = -t[K-2-j], middle boundary 0): the
// bucket is found on |y|, half the compares and selects.  With H = K / 2 magnitude buckets, a coordinate
// y >= 0 in magnitude bucket m has index H + m, a negative one H - 1 - m, i.e. the low planes are m resp. its
// complement and the top plane is the sign compare.  "On a boundary, the upper cell" means |y| >= T for y >= 0 but
// |y| > T for y < 0: negative coordinates are compared one ulp smaller (a subtract-with-borrow whose borrow is the
// sign mask).  An empty table (B = 0) is the generic case.
template <int B>
__device__ __forceinline__ float quantise_tile_sym(floatx16& acc, const float inv, const Codebook& cb, const int h,
                                                   uint32_t (&word)[4]) {
  if constexpr (B == 0) {
    return quantise_tile<0>(acc, inv, cb, h, word);
  } else {
    constexpr int H = 1 << (B - 1);
    float g2 = 0.f;
    uint32_t nib[4][B];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
#pragma unroll
      for (int pl = 0; pl < B; ++pl) nib[k][pl] = 0u;
#pragma unroll
      for (int r = 3; r >= 0; --r) {
        const float y = acc[4 * k + r] * inv;
        const uint64_t pos = __builtin_amdgcn_ballot_w64(y >= 0.f);  // -0 counts as 0: upper cell
        uint32_t ay = __float_as_uint(y) & 0x7fffffffu;
        {  // ay -= 1 where y < 0 (never for ay = 0: that is y = -0, which is in pos)
          uint64_t borrow_out;
          const uint64_t neg = ~pos;
          asm("v_subb_co_u32 %0, %1, %2, 0, %3" : "=v"(ay), "=s"(borrow_out) : "v"(ay), "s"(neg));
        }
        const float ayf = __uint_as_float(ay);
        float ym = cb.c[H];
        uint64_t mbit[B > 1 ? B - 1 : 1];
#pragma unroll
        for (int pl = 0; pl < (B > 1 ? B - 1 : 1); ++pl) mbit[pl] = 0;
#pragma unroll
        for (int j = 0; j < H - 1; ++j) {
          const float tj = cb.t[H + j], cj = cb.c[H + j + 1];  // read before the select, see quantise_tile
          const bool ge = ayf >= tj;
          ym = ge ? cj : ym;
          const uint64_t gem = __builtin_amdgcn_ballot_w64(ge);
#pragma unroll
          for (int pl = 0; pl < B - 1; ++pl)
            if ((j & ((1 << pl) - 1)) == (1 << pl) - 1) mbit[pl] ^= gem;
        }
        // the centroid takes the sign of y
        const float yt = __uint_as_float((__float_as_uint(ym) & 0x7fffffffu) | (__float_as_uint(y) & 0x80000000u));
        float e = y - yt;
        asm volatile("" : "+v"(e));
        g2 = fmaf(e, e, g2);
        acc[4 * k + r] = e;
#pragma unroll
        for (int pl = 0; pl < B - 1; ++pl) nib[k][pl] = shift_in(nib[k][pl], mbit[pl] ^ ~pos);
        nib[k][B - 1] = shift_in(nib[k][B - 1], pos);
      }
    }
#pragma unroll
    for (int pl = 0; pl < B; ++pl) {
      const uint32_t w = (nib[0][pl] | (nib[1][pl] << 8) | (nib[2][pl] << 16) | (nib[3][pl] << 24)) << (4 * h);
      word[pl] = or_across_halves(w);
    }
    return g2;
  }
}

// The cheaper of the two for a symmetric table: from 3 bits on the decision on |y| wins (C3 shape, 3 bits: 150 us
// against 167); at 1 and 2 bits its longer dependent chain per coordinate costs more than the two instructions it
// saves (2 bits: 140 us against 130).
template <int B>
__device__ __forceinline__ float quantise_tile_best(floatx16& acc, const float inv, const Codebook& cb, const int h,
                                                    uint32_t (&word)[4]) {
  if constexpr (B >= 3) return quantise_tile_sym<B>(acc, inv, cb, h, word);
  else return quantise_tile<B>(acc, inv, cb, h, word);
}

// c[i] == -c[K-1-i] and t[j] == -t[K-2-j] for a table of K = 2^bits entries (the middle boundary is then 0)
inline bool codebook_symmetric(const Codebook& cb, int bits) {
  const int K = 1 << bits;
  for (int i = 0; i < K; ++i)
    if (cb.c[i] != -cb.c[K - 1 - i]) return false;
  for (int j = 0; j + 1 < K; ++j)
    if (cb.t[j] != -cb.t[K - 2 - j]) return false;
  return true;
}

}  // namespace tq
