// In-kernel query preparation shared by the single-kernel d = 128 scoring kernels
// (tq_score_i8_128.hip, tq_score_i8_split.hip): a workgroup of 8 wavefronts rotates / sketches
// its own four queries from the transposed matrices and writes their balanced base-128 digits.
//
//   load      wavefront w requests its thread's column of matrix w / 4 (0: Pi^T, 1: S^T), half
//             (w / 2) % 2 of k, column j = tid % 128: 64 values, to be issued before anything else
//   matvec    y_j partial sums for the four queries (query coordinates through scalar
//             registers) -> part_s[matrix][half][query][j]
//   (barrier)
//   digitise  wavefront w takes (matrix w / 4, query w % 4): power-of-two scale with |Q| <= 2^19,
//             digits -> dig_s[matrix][query][digit][j] (digit 3 = 0), scalars -> scal_s[matrix][query]
//             [0: 1/scale, 1: sum of the rounded coordinates, 2: that sum over j < d_hi, 3: over the rest]
//   (barrier)
#pragma once
#include "tq_score_i8.h"

namespace tq {

// Slot of coordinate c (d = 128) among the 128 operand bytes of a digit row when the mask bytes are the stored
// bits left in place: k-step s = bit 2 of c, k-chunk kq = c / 32, dword i = c % 4, byte b = (c / 8) % 4.
__host__ __device__ constexpr int i8_shifted_slot(int c) {
  return (((c >> 2) & 1) * 4 + (c >> 5)) * 16 + (c & 3) * 4 + ((c >> 3) & 3);
}

constexpr int I8_PREP_BYTES = 2 * 2 * 4 * 128 * 4 + 2 * 4 * 4 * 128 + 2 * 4 * 4 * 4;  // partial sums, digits, scalars

// max / sum over the 64 lanes: four DPP steps inside each row of 16, then the four rows
// through scalar registers
template <int CTRL>
__device__ __forceinline__ int dpp_move(int v) {
  return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xF, 0xF, false);
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, __int_as_float(dpp_move<0xB1>(__float_as_int(v))));   // quad_perm [1,0,3,2]
  v = fmaxf(v, __int_as_float(dpp_move<0x4E>(__float_as_int(v))));   // quad_perm [2,3,0,1]
  v = fmaxf(v, __int_as_float(dpp_move<0x141>(__float_as_int(v))));  // row_half_mirror
  v = fmaxf(v, __int_as_float(dpp_move<0x140>(__float_as_int(v))));  // row_mirror
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
  const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
  const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
  return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}
__device__ __forceinline__ int wave_sum(int v) {
  v += dpp_move<0xB1>(v);
  v += dpp_move<0x4E>(v);
  v += dpp_move<0x141>(v);
  v += dpp_move<0x140>(v);
  return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
         __builtin_amdgcn_readlane(v, 48);
}

template <bool HAVE_R, bool PROD>
struct I8Prep {
  float wv[64];
  int mat, kh, j;
  bool work;

  __device__ __forceinline__ void load(const ScoreI8Args& a, int wave, int tid) {
    mat = wave >> 2;
    kh = (wave >> 1) & 1;
    j = tid & 127;
    work = mat == 0 ? HAVE_R : PROD;  // uniform
    if (work) {
      const float* WT = (mat ? a.ST : a.PiT) + (64 * kh) * 128 + j;
#pragma unroll
      for (int k = 0; k < 64; ++k) wv[k] = WT[k * 128];
    }
  }

  __device__ __forceinline__ void matvec(const ScoreI8Args& a, int group, int q0, float* part_s) {
    if (!work) return;
    const float* xq[4];  // uniform addresses: the query coordinates arrive in scalar registers
#pragma unroll
    for (int qi = 0; qi < 4; ++qi) {
      const int64_t r = (int64_t)group * a.q_per_group + (q0 + qi < a.q_per_group ? q0 + qi : q0);
      xq[qi] = a.x + r * a.ldx + 64 * kh;
    }
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < 64; ++k)
#pragma unroll
      for (int qi = 0; qi < 4; ++qi) acc[qi] = fmaf(wv[k], xq[qi][k], acc[qi]);
#pragma unroll
    for (int qi = 0; qi < 4; ++qi) part_s[((mat * 2 + kh) * 4 + qi) * 128 + j] = acc[qi];
  }

  // SHIFTED: the digit image for operands whose mask bytes are the stored bits left in place (bit k of a byte
  // reads as 2^k, as -128 for k = 7): coordinate c is written as Q 2^(7 - c % 8), negated where c % 8 = 7, in
  // four digits, at slot i8_shifted_slot(c); the masked sum of the products is then 128 times that of Q.
  template <bool SHIFTED = false>
  __device__ __forceinline__ static void digitise(const ScoreI8Args& a, int q0, int wave, int lane, int d_hi,
                                                  const float* part_s, signed char* dig_s, float* scal_s) {
    const int m = wave >> 2, qi = wave & 3;
    if (!(m == 0 ? HAVE_R : PROD)) return;
    const bool live = q0 + qi < a.q_per_group;
    float y[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int c = lane + 64 * u;
      y[u] = live ? part_s[((m * 2 + 0) * 4 + qi) * 128 + c] + part_s[((m * 2 + 1) * 4 + qi) * 128 + c] : 0.f;
    }
    const float mx = wave_max(fmaxf(fabsf(y[0]), fabsf(y[1])));
    int e = 0;
    if (mx > 0.f) (void)frexpf(mx, &e);  // mx = f * 2^e, f in [0.5, 1): |Q| <= 2^19
    const float sc = ldexpf(1.f, 19 - e);
    int Q[2];
    Q[0] = __float2int_rn(y[0] * sc);
    Q[1] = __float2int_rn(y[1] * sc);
    const int tot = wave_sum(Q[0] + Q[1]);
    const int tot_hi = wave_sum((lane < d_hi ? Q[0] : 0) + (lane + 64 < d_hi ? Q[1] : 0));
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      // balanced base 128: D0, D1 in [-64, 63], D2 in [-64, 64] (SHIFTED: D2 as D1, |D3| <= 33)
      const int c = lane + 64 * u, k = c & 7;
      const int Qs = !SHIFTED ? Q[u] : k == 7 ? -Q[u] : Q[u] << (7 - k);
      const int d0 = ((Qs + 64) & 127) - 64;
      const int Q1 = (Qs - d0) >> 7;
      const int d1 = ((Q1 + 64) & 127) - 64;
      const int Q2 = (Q1 - d1) >> 7;
      const int d2 = SHIFTED ? ((Q2 + 64) & 127) - 64 : Q2;
      const int d3 = (Q2 - d2) >> 7;
      signed char* o = dig_s + (m * 4 + qi) * 4 * 128 + (SHIFTED ? i8_shifted_slot(c) : c);
      o[0] = (signed char)d0;
      o[128] = (signed char)d1;
      o[256] = (signed char)d2;
      o[384] = (signed char)d3;
    }
    if (lane == 0) {
      const float inv = ldexpf(1.f, e - 19);
      scal_s[(m * 4 + qi) * 4 + 0] = inv;
      scal_s[(m * 4 + qi) * 4 + 1] = (float)tot * inv;
      scal_s[(m * 4 + qi) * 4 + 2] = (float)tot_hi * inv;
      scal_s[(m * 4 + qi) * 4 + 3] = (float)(tot - tot_hi) * inv;
    }
  }
};

// Four balanced base-128 digits of fixed-point value Q of coordinate c, in the shifted form (Q 2^(7 - c % 8), negated
// where c % 8 = 7) at slot i8_shifted_slot(c) of image `term`, query qi: dig_s[term][qi][digit][slot].
__device__ __forceinline__ void i8_put_shifted(signed char* dig_s, int term, int qi, int c, int Q) {
  const int k = c & 7;
  const int Qs = k == 7 ? -Q : Q << (7 - k);
  const int d0 = ((Qs + 64) & 127) - 64;
  const int Q1 = (Qs - d0) >> 7;
  const int d1 = ((Q1 + 64) & 127) - 64;
  const int Q2 = (Q1 - d1) >> 7;
  const int d2 = ((Q2 + 64) & 127) - 64;
  const int d3 = (Q2 - d2) >> 7;
  signed char* o = dig_s + (term * 4 + qi) * 4 * 128 + i8_shifted_slot(c);
  o[0] = (signed char)d0;
  o[128] = (signed char)d1;
  o[256] = (signed char)d2;
  o[384] = (signed char)d3;
}

__device__ __forceinline__ float wave_sum_f(float v) {
  v += __int_as_float(dpp_move<0xB1>(__float_as_int(v)));
  v += __int_as_float(dpp_move<0x4E>(__float_as_int(v)));
  v += __int_as_float(dpp_move<0x141>(__float_as_int(v)));
  v += __int_as_float(dpp_move<0x140>(__float_as_int(v)));
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0)) + __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16)) +
         __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32)) + __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
}

// Digit images for the d = 128 single-kernel path, one per masked sum, so that all the masked sums of the
// rotated query share ONE accumulator: term t (the t-th plane subset of odd size, factor coef[m]) is the image of
// Q = round(coef[m] y 2^s), s the power of two with max |coef| max |y| 2^s <= 2^19, in the shifted form of
// I8Prep::digitise<true>; the sketch term (index 2^(BITS-1)) is that of S q as before.  Wavefront w takes
// (matrix w / 4, query w % 4).
//   dig_s[term][query][digit][slot]; scal_s[matrix][query][0: 2^-s, 1: matrix 0: coef[0] sum_j y_j, matrix 1:
//   2^-s sum_j Q_j]
__host__ __device__ constexpr int i8_terms(int bits, bool prod) { return (bits > 0 ? 1 << (bits - 1) : 0) + (prod ? 1 : 0); }

template <int BITS, bool PROD>
__device__ __forceinline__ void i8_digitise_terms(const ScoreI8Args& a, int q0, int wave, int lane, const float* part_s,
                                                  signed char* dig_s, float* scal_s) {
  constexpr int NM = (1 << BITS) - 1;
  constexpr int NTM = BITS > 0 ? 1 << (BITS - 1) : 0;
  const int m = wave >> 2, qi = wave & 3;
  if (!(m == 0 ? BITS > 0 : PROD)) return;
  const bool live = q0 + qi < a.q_per_group;
  float y[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int c = lane + 64 * u;
    y[u] = live ? part_s[((m * 2 + 0) * 4 + qi) * 128 + c] + part_s[((m * 2 + 1) * 4 + qi) * 128 + c] : 0.f;
  }
  auto put = [&](int term, int u, int Q) { i8_put_shifted(dig_s, term, qi, lane + 64 * u, Q); };
  float cmax = 1.f;
  if (m == 0) {
    cmax = 0.f;
#pragma unroll
    for (int v = 1; v <= NM; ++v)
      if (i8_term(v)) cmax = fmaxf(cmax, fabsf(a.coef[v]));
  }
  const float mx = wave_max(fmaxf(fabsf(y[0]), fabsf(y[1]))) * cmax;
  int e = 0;
  if (mx > 0.f) (void)frexpf(mx, &e);  // mx = f * 2^e, f in [0.5, 1): |Q| <= 2^19
  const float sc = ldexpf(1.f, 19 - e), inv = ldexpf(1.f, e - 19);
  if (m == 1) {
    const int Q0 = __float2int_rn(y[0] * sc), Q1 = __float2int_rn(y[1] * sc);
    const int tot = wave_sum(Q0 + Q1);
    put(NTM, 0, Q0);
    put(NTM, 1, Q1);
    if (lane == 0) {
      scal_s[(4 + qi) * 4 + 0] = inv;
      scal_s[(4 + qi) * 4 + 1] = (float)tot * inv;
    }
  } else {
    int term = 0;
#pragma unroll
    for (int v = 1; v <= NM; ++v) {
      if (!i8_term(v)) continue;
      put(term, 0, __float2int_rn(a.coef[v] * y[0] * sc));
      put(term, 1, __float2int_rn(a.coef[v] * y[1] * sc));
      ++term;
    }
    const float ysum = wave_sum_f(y[0] + y[1]);
    if (lane == 0) {
      scal_s[qi * 4 + 0] = inv;
      scal_s[qi * 4 + 1] = a.coef[0] * ysum;
    }
  }
}

}  // namespace tq
