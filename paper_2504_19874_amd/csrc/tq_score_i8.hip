// Scoring for a few queries per code, integer-matrix-core version.
//
// The estimator of Sec. 3.2 in the rotated basis,
//     s = nu * ( sum_j qr_j c[idx_j]  +  kappa gamma sum_j qs_j z_j ),
// only ever multiplies query coordinates by a function of a few BITS of the
// code.  Written out over the bit planes b_p of idx (the packed layout stores
// exactly these planes),
//     c[idx] = sum over subsets S of planes of  coef_S * prod_{p in S} b_p ,
// (coef = Moebius transform of the centroid table), so
//     sum_j qr_j c[idx_j] = coef_0 * sum_j qr_j + sum_S coef_S * M_S,
//     M_S = sum of qr_j over the coordinates where all planes in S are 1,
// and likewise sum_j qs_j z_j = 2 * M_Z - sum_j qs_j with Z the qjl plane.
// Every M is a 0/1-masked sum: an int8 x int8 contraction on the matrix cores
// (v_mfma_i32_16x16x64_i8) between fixed-point digits of the queries and the
// mask expanded to one byte per bit.  Unlike fp32 MFMA, this does not compete
// with the vector ALU for the expansion work, and the expansion itself is one
// LDS lookup per 8 coordinates (byte -> 8 bytes) instead of per-coordinate
// bit fiddling.
//
// Fixed point: per query, Q_j = round(q_j * 2^e) with |Q_j| < 2^20, offset to
// q'_j = Q_j + 2^20 in [0, 2^21) and split into three 7-bit digits (0..127, so
// they are valid signed bytes).  Rows of the A operand: 4 queries x (3 digits +
// one row of ones); the ones row yields popcount(mask), which removes the
// offset: sum_j mask_j Q_j = D0 + 2^7 D1 + 2^14 D2 - 2^20 popcount.  Integer
// arithmetic is exact; the only rounding is that of q to 21 bits (relative
// 2^-20 of the query's largest coordinate), far inside the 1e-4 tolerance.
//
// Operand layout of v_mfma_i32_16x16x64_i8: A row / B column = lane % 16, the
// lane's 16 bytes are 16 values of k for k-chunk lane / 16 (any bijection of k
// works as long as A and B use the same one); D[4*(lane/16) + r][lane % 16] in
// register r.  With row = 4*query + digit a lane ends up holding the three
// digit sums and the popcount for ONE (query, key) pair.
#include "tq_internal.h"

namespace tq {

typedef int v4i __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// Query preparation for the int8 path: rotate / sketch one query per workgroup
// (y = W q for W = Pi or S), choose the fixed-point scale, and write the digit
// bytes in the order the scoring kernel's A operand wants them.
// grid (nq, 1 or 2 matrices), 128 threads; thread j owns output coordinate j.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(128) void prep_i8_kernel(const int d, const float* __restrict__ W0,
                                                      const float* __restrict__ W1,
                                                      const float* __restrict__ x, const int64_t ldx,
                                                      uint4* __restrict__ img, float* __restrict__ scal) {
  extern __shared__ __attribute__((aligned(16))) float prep_s[];  // x[d] then y[d]
  float* xs = prep_s;
  float* ys = prep_s + d;
  __shared__ float red_mx[2];
  __shared__ int red_tot[2];
  const int tid = threadIdx.x;
  const int64_t q = blockIdx.x;
  const int mat = blockIdx.y;
  const float* W = mat == 0 ? W0 : W1;
  for (int k = tid; k < d; k += 128) xs[k] = x[q * ldx + k];
  __syncthreads();
  float mx = 0.f;
  for (int j = tid; j < d; j += 128) {
    const float4* w4 = reinterpret_cast<const float4*>(W + (int64_t)j * d);
    const float4* x4 = reinterpret_cast<const float4*>(xs);
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll 8
    for (int k4 = 0; k4 < d / 4; ++k4) {
      const float4 w = w4[k4], v = x4[k4];
      a0 = fmaf(w.x, v.x, a0); a1 = fmaf(w.y, v.y, a1); a2 = fmaf(w.z, v.z, a2); a3 = fmaf(w.w, v.w, a3);
    }
    const float y = (a0 + a1) + (a2 + a3);
    ys[j] = y;
    mx = fmaxf(mx, fabsf(y));
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  if ((tid & 63) == 0) red_mx[tid >> 6] = mx;
  __syncthreads();
  mx = fmaxf(red_mx[0], red_mx[1]);
  // power-of-two scale with |Q| < 2^20
  int e = 0;
  if (mx > 0.f) (void)frexpf(mx, &e);  // mx = f * 2^e, f in [0.5, 1)
  const float sc = ldexpf(1.f, 19 - e);
  int tot = 0;
  for (int j = tid; j < d; j += 128) tot += __float2int_rn(ys[j] * sc);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) tot += __shfl_xor(tot, off);
  if ((tid & 63) == 0) red_tot[tid >> 6] = tot;
  __syncthreads();
  if (tid == 0) {
    scal[(q * 2 + mat) * 2 + 0] = ldexpf(1.f, e - 19);
    scal[(q * 2 + mat) * 2 + 1] = (float)(red_tot[0] + red_tot[1]) * ldexpf(1.f, e - 19);
  }
  const int ks = d >> 6;
  for (int u = tid; u < ks * 16; u += 128) {  // unit = (k-step s, digit dg, k-chunk kq)
    const int kq = u & 3, dg = (u >> 2) & 3, s = u >> 4;
    uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const int Q = __float2int_rn(ys[64 * s + 16 * kq + k] * sc);
      const uint32_t qp = (uint32_t)(Q + (1 << 20));
      const uint32_t byte = dg == 3 ? 1u : ((qp >> (7 * dg)) & 0x7Fu);
      w[k >> 2] |= byte << (8 * (k & 3));
    }
    img[((q * 2 + mat) * ks + s) * 16 + dg * 4 + kq] = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// Image of one query's A operand, written by prep_i8_kernel: for matrix m (0: Pi q, 1: S q),
// k-step s, digit row dg, k-chunk kq the 16 bytes of coordinates 64 s + 16 kq .. + 15.
//   bytes:   img[((q * 2 + m) * ks + s) * 16 + dg * 4 + kq]      (16-byte units)
//   scalars: scal[(q * 2 + m) * 2 + {0: 1/scale, 1: sum of the rounded coordinates}]
struct ScoreI8Args {
  const uint4* img;
  const float* scal;
  const uint32_t* idx;
  const uint32_t* qjl;
  const float* gamma;
  const float* norm;
  float* scores;
  int64_t lds;
  int64_t n;
  int d;
  int q_per_group;
  int keys_per_wg;
  float kappa;
  float coef[8];  // coef[S] for plane subsets S = 0 .. 2^BITS - 1
};

constexpr int I8_MAX_KS = 8;  // d <= 512

// KSM: compile-time bound on the number of 64-coordinate k-steps (register arrays)
template <int BITS, bool PROD, int KSM>
__global__ __launch_bounds__(256) void score_i8_kernel(const ScoreI8Args a) {
  __shared__ __attribute__((aligned(8))) uint2 expand_s[256];  // byte -> one byte per bit
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int col = lane & 15;   // key within a tile / row of A
  const int kq = lane >> 4;    // k-chunk; also the query whose sums this lane receives
  const int group = blockIdx.y;
  const int q0 = blockIdx.z * 4;
  const int d = a.d;
  const int ks = d >> 6;  // k-steps of 64 coordinates

  {
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      lo |= ((tid >> b) & 1u) << (8 * b);
      hi |= ((tid >> (b + 4)) & 1u) << (8 * b);
    }
    expand_s[tid] = make_uint2(lo, hi);
  }

  // ---- A operands: digits of this group's queries, kept in registers -----------------
  // lane = row + 16*kq, row = 4*query + digit; digit 3 is the row of ones
  const int a_query = col >> 2, a_digit = col & 3;
  const bool a_live = q0 + a_query < a.q_per_group;
  const int64_t qrow = (int64_t)group * a.q_per_group + q0 + (a_live ? a_query : 0);
  v4i ar[KSM], as_[KSM];
#pragma unroll
  for (int s = 0; s < KSM; ++s) {
    uint4 r = make_uint4(0, 0, 0, 0), z = make_uint4(0, 0, 0, 0);
    if (s < ks) {
      if (BITS > 0) r = a.img[((qrow * 2 + 0) * ks + s) * 16 + a_digit * 4 + kq];
      if (PROD) z = a.img[((qrow * 2 + 1) * ks + s) * 16 + a_digit * 4 + kq];
    }
    ar[s] = v4i{(int)r.x, (int)r.y, (int)r.z, (int)r.w};
    as_[s] = v4i{(int)z.x, (int)z.y, (int)z.z, (int)z.w};
  }
  // scale and coordinate sum of the query kq whose results this lane receives
  const bool q_live = q0 + kq < a.q_per_group;
  const int64_t orow = (int64_t)group * a.q_per_group + q0 + (q_live ? kq : 0);
  const float r_inv = a.scal[(orow * 2 + 0) * 2], r_sum = a.scal[(orow * 2 + 0) * 2 + 1];
  const float s_inv = PROD ? a.scal[(orow * 2 + 1) * 2] : 0.f, s_sum = PROD ? a.scal[(orow * 2 + 1) * 2 + 1] : 0.f;
  const bool out_live = q0 + kq < a.q_per_group;
  __syncthreads();

  const int words_per_row = (d >> 5) * BITS;
  const int qw_per_row = d >> 5;
  const int64_t gbase = (int64_t)group * a.n;
  const int half_shift = 16 * (kq & 1);  // this lane's 16 coordinates inside a 32-bit word
  const char* const table = reinterpret_cast<const char*>(expand_s);

  auto expand16 = [&](uint32_t w16) -> v4i {  // low 16 bits -> 16 bytes of 0/1
    const uint2 lo = *reinterpret_cast<const uint2*>(table + ((w16 << 3) & 0x7F8u));
    const uint2 hi = *reinterpret_cast<const uint2*>(table + ((w16 >> 5) & 0x7F8u));
    return v4i{(int)lo.x, (int)lo.y, (int)hi.x, (int)hi.y};
  };
  auto masked_sum = [&](const v4i& acc) -> float {  // D0 + 2^7 D1 + 2^14 D2 - 2^20 popcount
    return (float)(acc[0] + (acc[1] << 7) + (acc[2] << 14) - (acc[3] << 20));
  };

  // A wavefront takes 4 tiles of 16 keys per pass and requests all of their code words
  // before touching any: the kernel lives on bytes in flight, not on arithmetic.
  constexpr int TPP = 4;                // tiles per pass
  constexpr int NM = (1 << BITS) - 1;   // number of non-empty plane subsets
  constexpr int NW = BITS > 0 ? BITS : 1;
  const int64_t wg_key0 = (int64_t)blockIdx.x * a.keys_per_wg;
  const int passes = a.keys_per_wg / (4 * 16 * TPP);
  for (int pass = 0; pass < passes; ++pass) {
    const int64_t pass0 = wg_key0 + ((int64_t)pass * 4 + wave) * (16 * TPP);
    if (pass0 >= a.n) break;
    int64_t row[TPP];
    bool valid[TPP];
    uint32_t pw[TPP][KSM][NW], zw[TPP][KSM];
    float kg[TPP], nu[TPP];
#pragma unroll
    for (int t = 0; t < TPP; ++t) {
      const int64_t key = pass0 + t * 16 + col;
      valid[t] = key < a.n;
      row[t] = gbase + (valid[t] ? key : 0);
#pragma unroll
      for (int s = 0; s < KSM; ++s) {
        if (s >= ks) break;
        const int g = 2 * s + (kq >> 1);  // the 32-coordinate group this lane's k-chunk lies in
#pragma unroll
        for (int pl = 0; pl < BITS; ++pl) pw[t][s][pl] = a.idx[row[t] * words_per_row + g * BITS + pl];
        if (PROD) zw[t][s] = a.qjl[row[t] * qw_per_row + g];
      }
      kg[t] = PROD ? a.kappa * a.gamma[row[t]] : 0.f;
      nu[t] = a.norm != nullptr ? a.norm[row[t]] : 1.f;
    }
#pragma unroll
    for (int t = 0; t < TPP; ++t) {
      v4i acc[NM > 0 ? NM : 1], accz = {0, 0, 0, 0};
#pragma unroll
      for (int m = 0; m < (NM > 0 ? NM : 1); ++m) acc[m] = v4i{0, 0, 0, 0};
#pragma unroll
      for (int s = 0; s < KSM; ++s) {  // unrolled so the A registers are indexed statically
        if (s >= ks) break;
#pragma unroll
        for (int m = 1; m <= NM; ++m) {
          uint32_t w = 0xFFFFFFFFu;
#pragma unroll
          for (int pl = 0; pl < BITS; ++pl)
            if (m & (1 << pl)) w &= pw[t][s][pl];
          acc[m - 1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ar[s], expand16(w >> half_shift), acc[m - 1], 0, 0, 0);
        }
        if (PROD)
          accz = __builtin_amdgcn_mfma_i32_16x16x64_i8(as_[s], expand16(zw[t][s] >> half_shift), accz, 0, 0, 0);
      }
      float total = a.coef[0] * r_sum;
#pragma unroll
      for (int m = 1; m <= NM; ++m) total = fmaf(a.coef[m], masked_sum(acc[m - 1]) * r_inv, total);
      if (PROD) total = fmaf(kg[t], 2.f * masked_sum(accz) * s_inv - s_sum, total);
      total *= nu[t];
      if (valid[t] && out_live)
        a.scores[((int64_t)group * a.q_per_group + q0 + kq) * a.lds + pass0 + t * 16 + col] = total;
    }
  }
}

template <int BITS, bool PROD>
static hipError_t launch_ks(const ScoreI8Args& a, dim3 grid, hipStream_t s) {
  const int ks = a.d >> 6;
  if (ks <= 2)
    hipLaunchKernelGGL((score_i8_kernel<BITS, PROD, 2>), grid, dim3(256), 0, s, a);
  else if (ks <= 4)
    hipLaunchKernelGGL((score_i8_kernel<BITS, PROD, 4>), grid, dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL((score_i8_kernel<BITS, PROD, 8>), grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

template <int BITS>
static hipError_t launch_bits(const ScoreI8Args& a, bool prod, dim3 grid, hipStream_t s) {
  return prod ? launch_ks<BITS, true>(a, grid, s) : launch_ks<BITS, false>(a, grid, s);
}

size_t score_i8_workspace_bytes(int d, int64_t nq) {
  return (size_t)nq * 2 * ((size_t)(d >> 6) * 256 + 16) + 512;
}

hipError_t launch_score_i8(int bits, bool prod, const float* Pi, const float* S, const float* q, int64_t ldq,
                           void* workspace, const uint32_t* idx, const uint32_t* qjl, const float* gamma,
                           const float* norm, float* scores, int64_t lds, int64_t n, int d, int n_groups,
                           int q_per_group, float kappa, const Codebook& cb, hipStream_t stream) {
  if (n_groups == 0 || q_per_group == 0) return hipSuccess;
  if (bits < 0 || bits > 3 || d % 64 != 0 || d > 64 * I8_MAX_KS) return hipErrorInvalidValue;
  const int64_t nq = (int64_t)n_groups * q_per_group;
  uint4* img = static_cast<uint4*>(workspace);
  float* scal = reinterpret_cast<float*>(static_cast<char*>(workspace) + (size_t)nq * 2 * (d >> 6) * 256);
  hipLaunchKernelGGL(prep_i8_kernel, dim3((unsigned)nq, prod ? 2 : 1), dim3(128), (size_t)2 * d * sizeof(float),
                     stream, d, Pi, S, q, ldq, img, scal);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || n == 0) return e;
  ScoreI8Args a;
  a.img = img; a.scal = scal; a.idx = idx; a.qjl = qjl; a.gamma = gamma; a.norm = norm;
  a.scores = scores; a.lds = lds; a.n = n; a.d = d; a.q_per_group = q_per_group; a.kappa = kappa;
  // Moebius transform of the centroid table over the bit planes of the index
  double f[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  const int K = 1 << bits;
  for (int v = 0; v < K; ++v) f[v] = cb.c[v];
  for (int pl = 0; pl < bits; ++pl)
    for (int v = 0; v < K; ++v)
      if (v & (1 << pl)) f[v] -= f[v ^ (1 << pl)];
  for (int v = 0; v < 8; ++v) a.coef[v] = (float)f[v];
  // enough workgroups for every CU when the problem allows it, at least 64 keys per wavefront pass
  int64_t per_wg = 1024;  // a multiple of 256 = 4 wavefronts x 4 tiles x 16 keys
  while (per_wg > 256 && (n + per_wg - 1) / per_wg * n_groups < 1024) per_wg >>= 1;
  a.keys_per_wg = (int)per_wg;
  const dim3 grid((unsigned)((n + per_wg - 1) / per_wg), n_groups, (q_per_group + 3) / 4);
  switch (bits) {
    case 0: return launch_bits<0>(a, prod, grid, stream);
    case 1: return launch_bits<1>(a, prod, grid, stream);
    case 2: return launch_bits<2>(a, prod, grid, stream);
    case 3: return launch_bits<3>(a, prod, grid, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace tq
