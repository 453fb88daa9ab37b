// Few queries per code at d = 128 when the code is a pair of instances over a
// split of the rotated coordinates (Sec. 4.3: outlier channels with one more
// bit).  Coordinate group g < gs_hi (32 coordinates each) belongs to instance
// hi with BITS + 1 index planes and its own codebook, the others to instance lo
// with BITS planes; each instance has its own norm, residual norm and sketch
// scale, so the score is
//     nu_hi * (mse_hi + kappa_hi gamma_hi qjl_hi) + nu_lo * (mse_lo + kappa_lo gamma_lo qjl_lo)
// with the four inner sums taken over the instance's own coordinates only.
//
// Same arithmetic as tq_score_i8.hip (masked sums of fixed-point query digits on
// v_mfma_i32_16x16x64_i8, Walsh terms of the symmetric codebooks).  In that
// kernel's operand layout a lane's k-chunk IS one coordinate group, so "sum
// over one instance only" is an A operand with the other instance's lanes
// zeroed: every mask is expanded once and fed to two MFMAs, one per instance.
// Queries are prepared inside the kernel while the code words are in flight
// (FUSED, needs the transposed matrices; see tq_score_i8_prep.h), or by
// prep_i8_kernel beforehand; either leaves the per-instance sums of the rounded
// query coordinates.
#include "tq_score_i8_prep.h"

namespace tq {

struct SplitArgs {
  int gs_hi;
  float kappa_hi;   // sqrt(pi/2) / d_hi; ScoreI8Args::kappa is that of instance lo
  float coef_hi[16];  // Walsh form of the hi codebook; ScoreI8Args::coef is that of lo
};

constexpr int SPLIT_TILES = 8;  // tiles of 16 keys per wavefront

template <int BITS, bool PROD, bool FUSED>
__global__ __launch_bounds__(512) void score_i8_split_kernel(const ScoreI8Args a, const SplitArgs sp) {
  __shared__ __attribute__((aligned(16))) uint2 expand_s[256 * I8_COPIES];  // [256][32]: byte -> one byte per bit
  extern __shared__ __attribute__((aligned(16))) unsigned char prep_s[];   // FUSED: partial sums, digits, scalars
  float* const part_s = reinterpret_cast<float*>(prep_s);                               // [2][2][4][128]
  signed char* const dig_s = reinterpret_cast<signed char*>(part_s + 2 * 2 * 4 * 128);  // [2][4][4][128]
  float* const scal_s = reinterpret_cast<float*>(dig_s + 2 * 4 * 4 * 128);              // [2][4][4]
  constexpr int NP = BITS + 1;            // planes of instance hi
  constexpr int NMH = (1 << NP) - 1;      // plane subsets of hi
  constexpr int NML = (1 << BITS) - 1;    // plane subsets of lo (a prefix of hi's)
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 15;   // key within a tile / row of A
  const int kq = lane >> 4;    // k-chunk = coordinate group; also the query whose sums this lane receives
  const int group = blockIdx.y;
  const int q0 = blockIdx.z * 4;
  const int gs = sp.gs_hi;
  const bool g_hi = kq < gs;   // this lane's coordinate group belongs to instance hi

  // ---- A operands: digit images of this group's queries; one copy per instance ---------------
  const int a_query = col >> 2, a_digit = col & 3;
  const bool a_live = q0 + a_query < a.q_per_group;
  const int64_t qrow = (int64_t)group * a.q_per_group + q0 + (a_live ? a_query : 0);
  const bool out_live = q0 + kq < a.q_per_group;
  const int64_t orow = (int64_t)group * a.q_per_group + q0 + (out_live ? kq : 0);
  v4i ar[2][2], as_[2][2];  // [instance: 0 lo, 1 hi][k-step]
  float r_inv = 0.f, r_sum_hi = 0.f, r_sum_lo = 0.f, s_inv = 0.f, s_sum_hi = 0.f, s_sum_lo = 0.f;
  const v4i zero = v4i{0, 0, 0, 0};
  I8Prep<true, PROD> prep;
  if (FUSED) {
    prep.load(a, wave, tid);  // this thread's column of the transposed matrix, before anything else
  } else {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const uint4 r = a.img[((qrow * 2 + 0) * 2 + s) * 16 + a_digit * 4 + kq];
      const uint4 z = PROD ? a.img[((qrow * 2 + 1) * 2 + s) * 16 + a_digit * 4 + kq] : make_uint4(0, 0, 0, 0);
      const v4i rv = v4i{(int)r.x, (int)r.y, (int)r.z, (int)r.w}, zv = v4i{(int)z.x, (int)z.y, (int)z.z, (int)z.w};
      ar[1][s] = g_hi ? rv : zero;
      ar[0][s] = g_hi ? zero : rv;
      as_[1][s] = g_hi ? zv : zero;
      as_[0][s] = g_hi ? zero : zv;
    }
    r_inv = a.scal[(orow * 2 + 0) * 4];
    r_sum_hi = a.scal[(orow * 2 + 0) * 4 + 2];
    r_sum_lo = a.scal[(orow * 2 + 0) * 4 + 3];
    if (PROD) {
      s_inv = a.scal[(orow * 2 + 1) * 4];
      s_sum_hi = a.scal[(orow * 2 + 1) * 4 + 2];
      s_sum_lo = a.scal[(orow * 2 + 1) * 4 + 3];
    }
  }

  // ---- code words of this wavefront's keys: plane words of the lane's own group --------------
  const int wpr = 4 * BITS + gs;  // idx words per row
  const int woff = g_hi ? kq * NP : gs * NP + (kq - gs) * BITS;
  const int64_t gbase = (int64_t)group * a.n;
  const int64_t wave_key0 = ((int64_t)blockIdx.x * 8 + wave) * (16 * SPLIT_TILES);
  uint32_t pw[SPLIT_TILES][NP], zw[SPLIT_TILES];
  float kgh[SPLIT_TILES], kgl[SPLIT_TILES], nuh[SPLIT_TILES], nul[SPLIT_TILES];
#pragma unroll
  for (int t = 0; t < SPLIT_TILES; ++t) {
    const int64_t key = wave_key0 + t * 16 + col;
    const int64_t row = gbase + (key < a.n ? key : a.n - 1);  // clamped: results of such lanes are not stored
    const uint32_t* pi = a.idx + row * wpr + woff;
#pragma unroll
    for (int pl = 0; pl < BITS; ++pl) pw[t][pl] = pi[pl];
    pw[t][BITS] = g_hi ? pi[BITS] : 0u;  // a lo group has no such plane: an all-zero mask changes nothing
    zw[t] = PROD ? a.qjl[row * 4 + kq] : 0u;
    kgh[t] = PROD ? a.gamma[2 * row] : 0.f;
    kgl[t] = PROD ? a.gamma[2 * row + 1] : 0.f;
    nuh[t] = a.norm[2 * row];
    nul[t] = a.norm[2 * row + 1];
  }

  // ---- the expansion table, 32 bank-private copies ---------------------------------------------
  {
    const uint32_t lo = (((uint32_t)tid >> 5) * 0x00204081u) & 0x01010101u;  // bit i of the nibble -> byte i
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const uint32_t hi = ((uint32_t)i * 0x00204081u) & 0x01010101u;
      expand_s[tid + 512 * i] = make_uint2(lo, hi);
    }
  }
  if (FUSED) {
    prep.matvec(a, group, q0, part_s);
    __syncthreads();
    prep.digitise(a, q0, wave, lane, 32 * gs, part_s, dig_s, scal_s);
  }
  __syncthreads();
  if (FUSED) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int c0 = i8_coord0(s, kq);
      const v4i rv = *reinterpret_cast<const v4i*>(dig_s + ((0 * 4 + a_query) * 4 + a_digit) * 128 + c0);
      const v4i zv = PROD ? *reinterpret_cast<const v4i*>(dig_s + ((1 * 4 + a_query) * 4 + a_digit) * 128 + c0) : zero;
      ar[1][s] = g_hi ? rv : zero;
      ar[0][s] = g_hi ? zero : rv;
      as_[1][s] = g_hi ? zv : zero;
      as_[0][s] = g_hi ? zero : zv;
    }
    r_inv = scal_s[(0 * 4 + kq) * 4];
    r_sum_hi = scal_s[(0 * 4 + kq) * 4 + 2];
    r_sum_lo = scal_s[(0 * 4 + kq) * 4 + 3];
    if (PROD) {
      s_inv = scal_s[(1 * 4 + kq) * 4];
      s_sum_hi = scal_s[(1 * 4 + kq) * 4 + 2];
      s_sum_lo = scal_s[(1 * 4 + kq) * 4 + 3];
    }
  }

  const uint32_t copy_off = (uint32_t)(lane & (I8_COPIES - 1)) * 8u;
  const char* const table = reinterpret_cast<const char*>(expand_s);
  auto expand16 = [&](uint32_t w, int h) -> v4i {  // bits [16 h, 16 h + 16) of w -> 16 bytes of 0/1
    const uint32_t o0 = __builtin_amdgcn_perm(w, copy_off, h ? 0x0c0c0600u : 0x0c0c0400u);
    const uint32_t o1 = __builtin_amdgcn_perm(w, copy_off, h ? 0x0c0c0700u : 0x0c0c0500u);
    const uint2 lo = *reinterpret_cast<const uint2*>(table + o0);
    const uint2 hi = *reinterpret_cast<const uint2*>(table + o1);
    return v4i{(int)lo.x, (int)lo.y, (int)hi.x, (int)hi.y};
  };
  auto digits_sum = [&](const v4i& acc) -> float {  // D0 + 2^7 D1 + 2^14 D2
    return (float)(acc[0] + acc[1] * 128 + acc[2] * 16384);
  };

  // per-lane constants of the final combination
  float crh[NMH], crl[NML > 0 ? NML : 1];
#pragma unroll
  for (int m = 1; m <= NMH; ++m) crh[m - 1] = sp.coef_hi[m] * r_inv;
#pragma unroll
  for (int m = 1; m <= NML; ++m) crl[m - 1] = a.coef[m] * r_inv;
  const float base_hi = sp.coef_hi[0] * r_sum_hi, base_lo = a.coef[0] * r_sum_lo;
  const float zs = 2.f * s_inv;
  float* const out0 = a.scores + ((int64_t)group * a.q_per_group + q0 + kq) * a.lds + wave_key0 + col;

#pragma unroll
  for (int t = 0; t < SPLIT_TILES; ++t) {
    if (wave_key0 + t * 16 >= a.n) break;  // uniform over the wavefront
    v4i acch[NMH], accl[NML > 0 ? NML : 1], zh = {0, 0, 0, 0}, zl = {0, 0, 0, 0};
#pragma unroll
    for (int m = 0; m < NMH; ++m) acch[m] = v4i{0, 0, 0, 0};
#pragma unroll
    for (int m = 0; m < (NML > 0 ? NML : 1); ++m) accl[m] = v4i{0, 0, 0, 0};
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
      for (int m = 1; m <= NMH; ++m) {
        if (!i8_term(m)) continue;
        uint32_t w = 0u;
#pragma unroll
        for (int pl = 0; pl < NP; ++pl)
          if (m & (1 << pl)) w ^= pw[t][pl];
        const v4i b = expand16(w, s);
        acch[m - 1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ar[1][s], b, acch[m - 1], 0, 0, 0);
        if (m <= NML) accl[m - 1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ar[0][s], b, accl[m - 1], 0, 0, 0);
      }
      if (PROD) {
        const v4i b = expand16(zw[t], s);
        zh = __builtin_amdgcn_mfma_i32_16x16x64_i8(as_[1][s], b, zh, 0, 0, 0);
        zl = __builtin_amdgcn_mfma_i32_16x16x64_i8(as_[0][s], b, zl, 0, 0, 0);
      }
    }
    float th = base_hi, tl = base_lo;
#pragma unroll
    for (int m = 1; m <= NMH; ++m)
      if (i8_term(m)) th = fmaf(crh[m - 1], digits_sum(acch[m - 1]), th);
#pragma unroll
    for (int m = 1; m <= NML; ++m)
      if (i8_term(m)) tl = fmaf(crl[m - 1], digits_sum(accl[m - 1]), tl);
    if (PROD) {
      th = fmaf(sp.kappa_hi * kgh[t], fmaf(zs, digits_sum(zh), -s_sum_hi), th);
      tl = fmaf(a.kappa * kgl[t], fmaf(zs, digits_sum(zl), -s_sum_lo), tl);
    }
    const float total = fmaf(nuh[t], th, nul[t] * tl);
    if (out_live && wave_key0 + t * 16 + col < a.n) out0[t * 16] = total;
  }
}

template <int BITS, bool PROD, bool FUSED>
static hipError_t launch_split_one(const ScoreI8Args& a, const SplitArgs& sp, int n_groups, hipStream_t s) {
  const int64_t per_wg = 8 * 16 * SPLIT_TILES;
  const dim3 grid((unsigned)((a.n + per_wg - 1) / per_wg), n_groups, (a.q_per_group + 3) / 4);
  constexpr int lds = FUSED ? I8_PREP_BYTES : 0;  // on top of the 64 KB table
  static LdsLimit lds_limit;  // per instantiation: the limit is raised once per device
  if (FUSED) if (const hipError_t e = raise_lds_limit(lds_limit, reinterpret_cast<const void*>(&score_i8_split_kernel<BITS, PROD, FUSED>), lds); e != hipSuccess) return e;
  hipLaunchKernelGGL((score_i8_split_kernel<BITS, PROD, FUSED>), grid, dim3(512), lds, s, a, sp);
  return hipGetLastError();
}

template <int BITS, bool PROD>
static hipError_t launch_split(const ScoreI8Args& a, const SplitArgs& sp, int n_groups, bool fused, hipStream_t s) {
  return fused ? launch_split_one<BITS, PROD, true>(a, sp, n_groups, s) : launch_split_one<BITS, PROD, false>(a, sp, n_groups, s);
}

// c[v] = sum_S w_S chi_S(v) rewritten over masked sums (see tq_score_i8.hip):
//   sum_j q_j c[idx_j] = (w_0 - sum_S sgn_S w_S) * sum_j q_j + sum_S 2 sgn_S w_S M_S
static bool walsh_coefficients(int bits, const Codebook& cb, float* coef) {
  double w[16];
  i8_walsh(bits, cb, w);
  const int K = 1 << bits;
  double c0 = w[0];
  for (int v = 0; v < 16; ++v) coef[v] = 0.f;
  for (int sset = 1; sset < K; ++sset) {
    const double sgn = (__builtin_popcount(sset) & 1) ? 1.0 : -1.0;
    if (!i8_term(sset) && w[sset] != 0.0) return false;  // not symmetric about zero
    c0 -= sgn * w[sset];
    coef[sset] = (float)(2.0 * sgn * w[sset]);
  }
  coef[0] = (float)c0;
  return true;
}

bool score_i8_split_applicable(int bits_lo, const Codebook& cb_lo, const Codebook& cb_hi) {
  float tmp[16];
  return bits_lo >= 0 && bits_lo <= 3 && cb_hi.bits == bits_lo + 1 && walsh_coefficients(bits_lo, cb_lo, tmp) &&
         walsh_coefficients(bits_lo + 1, cb_hi, tmp);
}

hipError_t launch_score_i8_split(int bits_lo, bool prod, const float* Pi, const float* S, const float* PiT,
                                 const float* ST, const float* q, int64_t ldq,
                                 void* workspace, const uint32_t* idx, const uint32_t* qjl, const float* gamma,
                                 const float* norm, float* scores, int64_t lds, int64_t n, int n_groups,
                                 int q_per_group, int gs_hi, float kappa_lo, float kappa_hi, const Codebook& cb_lo,
                                 const Codebook& cb_hi, hipStream_t stream) {
  if (n_groups == 0 || q_per_group == 0 || n == 0) return hipSuccess;
  if (gs_hi < 1 || gs_hi > 3 || bits_lo < 0 || bits_lo > 3) return hipErrorInvalidValue;
  const int64_t nq = (int64_t)n_groups * q_per_group;
  uint4* img = static_cast<uint4*>(workspace);
  float* scal = reinterpret_cast<float*>(static_cast<char*>(workspace) + (size_t)nq * 2 * 2 * 256);
  // with the transposed matrices at hand the scoring kernel prepares the queries itself
  const bool fused = PiT != nullptr && (!prod || ST != nullptr);
  if (!fused) {
    hipError_t e = launch_prep_i8_128(32 * gs_hi, Pi, S, q, ldq, nq, prod, img, scal, stream);
    if (e != hipSuccess) return e;
  }
  ScoreI8Args a;
  a.img = img; a.scal = scal; a.PiT = PiT; a.ST = ST; a.x = q; a.ldx = ldq; a.idx = idx; a.qjl = qjl;
  a.gamma = gamma; a.norm = norm; a.scores = scores; a.lds = lds; a.n = n; a.total_rows = (int64_t)n_groups * n;
  a.d = 128; a.q_per_group = q_per_group; a.kappa = kappa_lo;
  SplitArgs sp;
  sp.gs_hi = gs_hi;
  sp.kappa_hi = kappa_hi;
  if (!walsh_coefficients(bits_lo, cb_lo, a.coef) || !walsh_coefficients(bits_lo + 1, cb_hi, sp.coef_hi))
    return hipErrorInvalidValue;
  switch (bits_lo * 2 + (prod ? 1 : 0)) {
    case 0: return launch_split<0, false>(a, sp, n_groups, fused, stream);
    case 1: return launch_split<0, true>(a, sp, n_groups, fused, stream);
    case 2: return launch_split<1, false>(a, sp, n_groups, fused, stream);
    case 3: return launch_split<1, true>(a, sp, n_groups, fused, stream);
    case 4: return launch_split<2, false>(a, sp, n_groups, fused, stream);
    case 5: return launch_split<2, true>(a, sp, n_groups, fused, stream);
    case 6: return launch_split<3, false>(a, sp, n_groups, fused, stream);
    case 7: return launch_split<3, true>(a, sp, n_groups, fused, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace tq
