// Attention read-out at d = 128 (see tq_attend.hip for the decomposition): the softmax-weighted
// sum of decoded value codes on the integer matrix cores.
//
// With a centroid table symmetric about zero, c[idx] = coef[0] + sum over the odd-sized plane
// subsets S of coef[S] * x_S(idx), x_S = XOR of the index bits in S (tq_score_i8.hip).  So for
// every query q and coordinate j
//     sum_i w_qi c[idx_ij] = coef[0] * sum_i w_qi + sum_S coef[S] * sum_i w_qi x_S(idx_ij):
// sums of weights over the KEYS selected by a bit mask.  The sign term of Alg. 2 is one more
// such sum, over the sign bits with the weights exp(logit - m) * nu_i * gamma_i (VPROD).  The weights w_qi = exp(logit - m) * nu_i
// are scaled by a power of two to 26-bit integers and split into four base-128 digits (0..127);
// one v_mfma_i32_16x16x64_i8 multiplies the 16 rows (4 queries x 4 digits) with 64 keys x 16
// coordinates of 0/1 bytes.
//
// The contraction runs over keys, but a code word holds 32 COORDINATES of one key.  Each lane
// therefore takes the words of 16 keys (one coordinate group, one plane) and transposes the
// 16 x 32 bit block in registers (two 16 x 16 transposes side by side in the halves of a 32-bit
// register); the transposed words go through LDS to the lanes that need them as B operands, which
// expand 16 bits (16 keys of one coordinate) to 16 bytes through a 256-entry table, as the scoring
// kernels do.
//
// Workgroup of 8 wavefronts = 2048 keys of one group, 4 queries; a wavefront owns 256 consecutive
// keys and takes 128 per pass.  Per pass and wavefront: 2 k-blocks of 64 keys x 8 coordinate
// blocks x terms MFMAs.
//
// FUSED: the logits come from the d = 128 scoring kernel run in place (tq_score_i8_128_body.h: the
// lane of (query, key) keeps its score in a register), so neither a score nor a dequantised
// value ever reaches memory.  Otherwise they are read from a score matrix computed beforehand
// (key codes the scoring body does not take).
#pragma once
#include "tq_attend.h"
#include "tq_score_i8_128_body.h"

#include <type_traits>

namespace tq {

constexpr int AT_WAVE_KEYS = 256;                    // keys a wavefront owns
constexpr int AT_PASS_KEYS = 128;                    // ... and handles per pass
constexpr int AT_PASSES = AT_WAVE_KEYS / AT_PASS_KEYS;
constexpr int AT_CHUNK = 8 * AT_WAVE_KEYS;
constexpr int AT_WD_BYTES = 8 * 4 * 4 * AT_PASS_KEYS;  // weight digits [wave][query][digit][key]
constexpr int AT_XCH_BYTES = 8 * 8 * 64 * 4;            // per plane: [wave][block of 16 keys][64 words]
constexpr int AT_RED_FLOATS = 3 * 8 * 4;  // [maxima | norm maxima | sums][wave][4]

// dynamic LDS: digits, exchange area (or, before them in time, what the scoring body needs), then the
// reduction scratch, which is written while other wavefronts may still be scoring
// (two: a second set of weight digits and one more plane: the signs of Alg. 2, or the top plane of instance hi)
__host__ __device__ constexpr int attend128_work_bytes(int kb, int vb, bool two, bool fused) {
  const int own = (two ? 2 : 1) * AT_WD_BYTES + (vb + (two ? 1 : 0)) * AT_XCH_BYTES;
  return fused && score128_lds(kb) > own ? score128_lds(kb) : own;
}
__host__ __device__ constexpr int attend128_lds(int kb, int vb, bool two, bool fused) {
  return attend128_work_bytes(kb, vb, two, fused) + AT_RED_FLOATS * 4;
}

struct AttendCoefs {
  float c[16];
};

// max / sum over the 16 lanes of a row (lanes sharing lane / 16); every lane receives the result
__device__ __forceinline__ float row_max(float v) {
  v = fmaxf(v, __int_as_float(dpp_move<0xB1>(__float_as_int(v))));
  v = fmaxf(v, __int_as_float(dpp_move<0x4E>(__float_as_int(v))));
  v = fmaxf(v, __int_as_float(dpp_move<0x141>(__float_as_int(v))));
  v = fmaxf(v, __int_as_float(dpp_move<0x140>(__float_as_int(v))));
  return v;
}
__device__ __forceinline__ float row_sum(float v) {
  v += __int_as_float(dpp_move<0xB1>(__float_as_int(v)));
  v += __int_as_float(dpp_move<0x4E>(__float_as_int(v)));
  v += __int_as_float(dpp_move<0x141>(__float_as_int(v)));
  v += __int_as_float(dpp_move<0x140>(__float_as_int(v)));
  return v;
}

// x[i] bit c (16 rows, 32 columns)  ->  x[c'] bit t = old x[t] bit c' and x[c'] bit 16 + t = old x[t] bit 16 + c':
// two 16 x 16 transposes, one in each half of the registers
__device__ __forceinline__ void transpose16x32(uint32_t (&x)[16]) {
#define TQ_SWAP_STAGE(J, M)                                      \
  _Pragma("unroll") for (int k = 0; k < 16; ++k) if (!(k & J)) { \
    const uint32_t a = x[k], b = x[k + J];                       \
    x[k + J] = ((a >> J) & M) | (b & ~M);                        \
    x[k] = (a & ~(M << J)) | ((b << J) & (M << J));              \
  }
  TQ_SWAP_STAGE(8, 0x00FF00FFu)
  TQ_SWAP_STAGE(4, 0x0F0F0F0Fu)
  TQ_SWAP_STAGE(2, 0x33333333u)
  TQ_SWAP_STAGE(1, 0x55555555u)
#undef TQ_SWAP_STAGE
}

// ka: arguments of the scoring body (FUSED only); a: value codes, partial results, and with !FUSED the score matrix
// VKIND, the kind of value code: 0 = Alg. 1; 1 = Alg. 2 (one more plane: the signs, with weights ... * gamma);
// 2 = two instances of Alg. 1 over a split of the coordinates (Sec. 4.3): groups g < a.gs_hi have VB + 1 index
// planes, the table cfh and the weights exp(.) * nu_hi, the others VB planes, cf and exp(.) * nu_lo.
template <int KB, bool KPROD, int VB, int VKIND, bool FUSED>
__global__ __launch_bounds__(512) void attend128_kernel(const ScoreI8Args ka, const AttendArgs a, const AttendCoefs cf,
                                                        const AttendCoefs cfh) {
  constexpr bool VPROD = VKIND == 1, VSPLIT = VKIND == 2, TWO = VKIND != 0;  // TWO: a second set of weights
  __shared__ __attribute__((aligned(16))) uint2 expand_s[256 * I8_COPIES];  // byte -> one byte per bit, 32 copies
  extern __shared__ __attribute__((aligned(16))) unsigned char dyn_s[];
  constexpr int NPL = VB + (TWO ? 1 : 0);  // bit planes of a value code: index planes, then the signs of Alg. 2 / the top plane of instance hi
  constexpr int NVB = VB > 0 ? VB : 1;
  constexpr int ROUNDS = (NPL + 1) / 2;       // planes a transposing lane takes: ph, ph + 2
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 15;  // key within a tile; B column (coordinate within a block of 16); A row (query, digit)
  const int kc = lane >> 4;   // query of this lane's logits and sums; k-chunk (16 keys of a k-block)
  const int chunk = blockIdx.x, group = blockIdx.y, q0 = blockIdx.z * 4;
  constexpr int WD_ALL = (TWO ? 2 : 1) * AT_WD_BYTES;
  unsigned char* const wd = dyn_s + wave * (4 * 4 * AT_PASS_KEYS);  // digits of exp(.) nu; + AT_WD_BYTES: of exp(.) nu gamma
  uint32_t* const xch = reinterpret_cast<uint32_t*>(dyn_s + WD_ALL) + wave * (8 * 64);  // + plane * 8 * 8 * 64
  float* const fsum_s = reinterpret_cast<float*>(dyn_s + WD_ALL);  // [8][4][128], over the exchange area
  float* const fsumz_s = reinterpret_cast<float*>(dyn_s);          // the same for the sign sums, over the digits
  float* const red_s = reinterpret_cast<float*>(dyn_s + attend128_work_bytes(KB, VB, TWO, FUSED));  // [3][8][4]

  const int64_t gbase = (int64_t)group * a.group_stride;
  const int64_t wave_key0 = ((int64_t)chunk * 8 + wave) * AT_WAVE_KEYS;
  // transposing role: block kb of 16 keys, coordinate group tg, planes ph and ph + 2
  const int kb = lane & 7, tg = (lane >> 3) & 3, ph = lane >> 5;

  uint32_t vw[ROUNDS][16];
  auto load_codes = [&](int ps) {
    const int64_t k0 = wave_key0 + ps * AT_PASS_KEYS + 16 * kb;
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
      const int plane = ph + 2 * r;
      // an odd number of planes: the last round has work for half the lanes only
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int64_t key = k0 + i;
        const int64_t row = gbase + (key < a.n ? key : a.n - 1);  // clamped: such keys have weight 0
        if (VSPLIT) {
          const bool thi = tg < a.gs_hi;
          const int wpr = 4 * VB + a.gs_hi, woff = thi ? tg * (VB + 1) : a.gs_hi + tg * VB;
          vw[r][i] = plane < VB + (thi ? 1 : 0) ? a.idx[row * wpr + woff + plane] : 0u;  // no such plane: all-zero mask
        } else {
          vw[r][i] = plane < VB ? a.idx[row * (4 * VB) + tg * VB + plane] : (VPROD && plane == VB) ? a.qjl[row * 4 + tg] : 0u;
        }
      }
    }
  };

  // value norms: lane L holds those of keys L, L + 64, L + 128, L + 192 of the wavefront
  // (and nu gamma, the factor of the sign term of Alg. 2)
  float nuv[4], ngv[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int64_t key = wave_key0 + 64 * e + lane;
    if (VSPLIT) {  // (nu_hi, nu_lo) per token
      nuv[e] = key < a.n ? a.norm[2 * (gbase + key) + 1] : 0.f;
      ngv[e] = key < a.n ? a.norm[2 * (gbase + key)] : 0.f;
    } else {
      nuv[e] = key < a.n ? a.norm[gbase + key] : 0.f;
      ngv[e] = VPROD && key < a.n ? nuv[e] * a.gamma[gbase + key] : 0.f;
    }
  }
  // the first pass's value codes travel while the keys are scored, where the registers allow it
  constexpr bool EARLY = !FUSED || KB + (KPROD ? 1 : 0) <= 4;
  if (EARLY) load_codes(0);

  // ---- logits: lane (kc, col) holds those of (query q0 + kc, key wave_key0 + 16 t + col), t < 16 ----
  // (kept in units of log 2, so that the weights are one v_exp_f32 each)
  float lg[16];
  const float scale2 = a.scale * 1.44269504088896341f;
#pragma unroll
  for (int t = 0; t < 16; ++t) lg[t] = -INFINITY;
  if (FUSED) {
    auto sink = [&](int t, float score, bool key_live) { lg[t] = key_live ? scale2 * score : -INFINITY; };
    score128_body<KB, KPROD, TILES_128, SCORE128_ROUND_TILES, SCORE128_ROUNDS_AHEAD>(ka, dyn_s, sink);
  } else {
    const int64_t qrow = (int64_t)group * a.q_per_group + (q0 + kc < a.q_per_group ? q0 + kc : q0);
    const float* srow = a.scores + qrow * a.lds + wave_key0 + col;
#pragma unroll
    for (int t = 0; t < 16; ++t)
      if (wave_key0 + 16 * t + col < a.n) lg[t] = scale2 * srow[16 * t];
  }
  {
    const uint32_t lo = (((uint32_t)tid >> 5) * 0x00204081u) & 0x01010101u;  // the expansion table of the read-out
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const uint32_t hi = ((uint32_t)i * 0x00204081u) & 0x01010101u;
      expand_s[tid + 512 * i] = make_uint2(lo, hi);
    }
  }
  if (!EARLY) load_codes(0);

  // ---- chunk maxima: logits per query, value norm ---------------------------------------------
  {
    float v = lg[0];
#pragma unroll
    for (int t = 1; t < 16; ++t) v = fmaxf(v, lg[t]);
    v = row_max(v);
    if (col == 0) red_s[wave * 4 + kc] = v;
    const float nm = wave_max(fmaxf(fmaxf(nuv[0], nuv[1]), fmaxf(nuv[2], nuv[3])));
    if (lane == 1) red_s[32 + wave * 4] = nm;
    if (TWO) {
      const float gm = wave_max(fmaxf(fmaxf(ngv[0], ngv[1]), fmaxf(ngv[2], ngv[3])));
      if (lane == 2) red_s[32 + wave * 4 + 1] = gm;
    }
  }
  __syncthreads();  // also: every wavefront is done with the scoring body's LDS
  float m = -INFINITY, numax = 0.f, ngmax = 0.f;
#pragma unroll
  for (int w = 0; w < 8; ++w) {
    m = fmaxf(m, red_s[w * 4 + kc]);
    numax = fmaxf(numax, red_s[32 + w * 4]);
    if (TWO) ngmax = fmaxf(ngmax, red_s[32 + w * 4 + 1]);
  }
  int enu = 0, eng = 0;
  if (numax > 0.f) (void)frexpf(numax, &enu);  // numax = f * 2^enu, f in [0.5, 1)
  if (ngmax > 0.f) (void)frexpf(ngmax, &eng);
  const float wscale = ldexpf(1.f, 26 - enu);  // weights exp(logit - m) * nu * wscale <= 2^26
  const float zscale = ldexpf(1.f, 26 - eng);

  const uint32_t copy_off = (uint32_t)(lane & (I8_COPIES - 1)) * 8u;
  const char* const table = reinterpret_cast<const char*>(expand_s);
  auto expand16 = [&](uint32_t w, int h) -> v4i {  // bits [16 h, 16 h + 16) of w -> 16 bytes of 0/1
    const uint32_t o0 = __builtin_amdgcn_perm(w, copy_off, h ? 0x0c0c0600u : 0x0c0c0400u);
    const uint32_t o1 = __builtin_amdgcn_perm(w, copy_off, h ? 0x0c0c0700u : 0x0c0c0500u);
    const uint2 lo = *reinterpret_cast<const uint2*>(table + o0);
    const uint2 hi = *reinterpret_cast<const uint2*>(table + o1);
    return v4i{(int)lo.x, (int)lo.y, (int)hi.x, (int)hi.y};
  };
  auto digits_sum = [&](const v4i& acc) -> float {  // D0 + 2^7 D1 + 2^14 D2 + 2^21 D3
    return fmaf((float)acc[3], 2097152.f, (float)(acc[0] + acc[1] * 128 + acc[2] * 16384));
  };

  float f[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};  // coordinate 16 cb + col of query kc
  float ftot = 0.f;                                         // sum of the integer weights of query kc
  float fz[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};  // VPROD: the same two for the weights of the sign term
  float fztot = 0.f;
  float lsum = 0.f;
  const v4i ones = v4i{0x01010101, 0x01010101, 0x01010101, 0x01010101};

#pragma unroll
  for (int ps = 0; ps < AT_PASSES; ++ps) {
    // weights of this lane's (query, key) pairs -> four base-128 digits
#pragma unroll
    for (int tt = 0; tt < 8; ++tt) {
      const int t = 8 * ps + tt;
      const float nu = __int_as_float(__builtin_amdgcn_ds_bpermute(4 * (16 * (t & 3) + col), __float_as_int(nuv[t >> 2])));
      const float p = __builtin_amdgcn_exp2f(lg[t] - m);  // 0 for keys past the end (logit -inf)
      lsum += p;
      // the weight is not negative: plain base-128 digits 0..127 fit the signed bytes of the operand
      const uint32_t Q = (uint32_t)__float2int_rn(p * nu * wscale);
      unsigned char* o = wd + (kc * 4) * AT_PASS_KEYS + 16 * tt + col;
      o[0] = (unsigned char)(Q & 127u);
      o[AT_PASS_KEYS] = (unsigned char)((Q >> 7) & 127u);
      o[2 * AT_PASS_KEYS] = (unsigned char)((Q >> 14) & 127u);
      o[3 * AT_PASS_KEYS] = (unsigned char)(Q >> 21);
      if (TWO) {
        const float ng = __int_as_float(__builtin_amdgcn_ds_bpermute(4 * (16 * (t & 3) + col), __float_as_int(ngv[t >> 2])));
        const uint32_t Z = (uint32_t)__float2int_rn(p * ng * zscale);
        o[AT_WD_BYTES] = (unsigned char)(Z & 127u);
        o[AT_WD_BYTES + AT_PASS_KEYS] = (unsigned char)((Z >> 7) & 127u);
        o[AT_WD_BYTES + 2 * AT_PASS_KEYS] = (unsigned char)((Z >> 14) & 127u);
        o[AT_WD_BYTES + 3 * AT_PASS_KEYS] = (unsigned char)(Z >> 21);
      }
    }
    // value code words: 16 keys x 32 coordinates -> 32 coordinates x 16 keys
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
      const int plane = ph + 2 * r;
      transpose16x32(vw[r]);
      if (plane < NPL) {
        // word c: low half = coordinate 32 tg + c, high half = coordinate 32 tg + 16 + c.  Odd key blocks swap
        // the halves of a row of 32 words, which keeps the reads below free of bank conflicts.
        uint4* dst = reinterpret_cast<uint4*>(xch + plane * (8 * 8 * 64) + kb * 64 + ((tg ^ (kb & 1)) * 16));
#pragma unroll
        for (int c = 0; c < 4; ++c) dst[c] = make_uint4(vw[r][4 * c], vw[r][4 * c + 1], vw[r][4 * c + 2], vw[r][4 * c + 3]);
      }
    }
    if (ps + 1 < AT_PASSES) load_codes(ps + 1);
    __syncthreads();

    v4i aop[2], zop[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      aop[kk] = *reinterpret_cast<const v4i*>(wd + col * AT_PASS_KEYS + kk * 64 + kc * 16);
      if (TWO) zop[kk] = *reinterpret_cast<const v4i*>(wd + AT_WD_BYTES + col * AT_PASS_KEYS + kk * 64 + kc * 16);
    }
    {
      v4i tot = v4i{0, 0, 0, 0}, ztot = v4i{0, 0, 0, 0};
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        tot = __builtin_amdgcn_mfma_i32_16x16x64_i8(aop[kk], ones, tot, 0, 0, 0);
        if (TWO) ztot = __builtin_amdgcn_mfma_i32_16x16x64_i8(zop[kk], ones, ztot, 0, 0, 0);
      }
      ftot += digits_sum(tot);
      if (TWO) fztot += digits_sum(ztot);
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      constexpr int NPW = VSPLIT ? VB + 1 : NVB;  // index planes read (instance lo: the top one is all zero)
      uint32_t pw[2][NPW], pz[2] = {0u, 0u};
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
        for (int pl = 0; pl < (VSPLIT ? VB + 1 : VB); ++pl)
          pw[kk][pl] = xch[pl * (8 * 8 * 64) + (4 * kk + kc) * 64 + ((g ^ (kc & 1)) * 16) + col];
        if (VPROD) pz[kk] = xch[VB * (8 * 8 * 64) + (4 * kk + kc) * 64 + ((g ^ (kc & 1)) * 16) + col];
      }
      // masked sums of one coordinate group: plane subsets of odd size, weights and table of the group's instance
      auto terms = [&](auto planes_c, const v4i (&wop)[2], const AttendCoefs& tab) {
        constexpr int NP = decltype(planes_c)::value;
#pragma unroll
        for (int mset = 1; mset < (1 << NP); ++mset) {
          if (!i8_term(mset)) continue;
          uint32_t mk[2] = {0u, 0u};
#pragma unroll
          for (int pl = 0; pl < NP; ++pl)
            if (mset & (1 << pl)) {
              mk[0] ^= pw[0][pl];
              mk[1] ^= pw[1][pl];
            }
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            v4i acc = v4i{0, 0, 0, 0};
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(wop[kk], expand16(mk[kk], h), acc, 0, 0, 0);
            f[2 * g + h] = fmaf(tab.c[mset], digits_sum(acc), f[2 * g + h]);
          }
        }
      };
      if (VSPLIT && g < a.gs_hi) terms(std::integral_constant<int, VB + 1>{}, zop, cfh);  // uniform
      else terms(std::integral_constant<int, VB>{}, aop, cf);
      if (VPROD) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          v4i acc = v4i{0, 0, 0, 0};
#pragma unroll
          for (int kk = 0; kk < 2; ++kk) acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(zop[kk], expand16(pz[kk], h), acc, 0, 0, 0);
          fz[2 * g + h] += digits_sum(acc);
        }
      }
    }
    __syncthreads();  // the digit and exchange areas are rewritten by the next pass / the final sums
  }

  // ---- join the wavefronts ------------------------------------------------------------------------
  lsum = row_sum(lsum);
  if (col == 0) red_s[64 + wave * 4 + kc] = lsum;
#pragma unroll
  for (int cb = 0; cb < 8; ++cb) {
    if (VSPLIT)  // each instance has its own table, weight total and weight scale
      fsum_s[(wave * 4 + kc) * 128 + 16 * cb + col] = (cb >> 1) < a.gs_hi ? fmaf(cfh.c[0], fztot, f[cb]) * ldexpf(1.f, eng - 26)
                                                                           : fmaf(cf.c[0], ftot, f[cb]) * ldexpf(1.f, enu - 26);
    else
      fsum_s[(wave * 4 + kc) * 128 + 16 * cb + col] = fmaf(cf.c[0], ftot, f[cb]);
    // sum of w z over the keys, z = +-1 from the sign bits: twice the masked sum minus the sum of the weights
    if (VPROD) fsumz_s[(wave * 4 + kc) * 128 + 16 * cb + col] = fmaf(2.f, fz[cb], -fztot);
  }
  __syncthreads();
  const int qi = tid >> 7, j = tid & 127;
  if (q0 + qi < a.q_per_group) {
    float acc = 0.f, accz = 0.f;
#pragma unroll
    for (int w = 0; w < 8; ++w) {
      acc += fsum_s[(w * 4 + qi) * 128 + j];
      if (VPROD) accz += fsumz_s[(w * 4 + qi) * 128 + j];
    }
    float* o = a.part + (((int64_t)group * a.q_per_group + q0 + qi) * a.nchunks + chunk) * attend_part_stride(128);
    o[4 + j] = VSPLIT ? acc : acc * ldexpf(1.f, enu - 26);
    o[4 + 128 + j] = VPROD ? accz * ldexpf(1.f, eng - 26) : 0.f;
    if (j == 0) {
      float l = 0.f, mq = -INFINITY;
#pragma unroll
      for (int w = 0; w < 8; ++w) {
        l += red_s[64 + w * 4 + qi];
        mq = fmaxf(mq, red_s[w * 4 + qi]);
      }
      o[0] = mq * 0.693147180559945309f;  // back to natural units
      o[1] = l;
    }
  }
}

template <int KB, bool KPROD, int VB, int VKIND, bool FUSED>
hipError_t launch_attend128_one(const ScoreI8Args& ka, const AttendArgs& a, const AttendCoefs& cf, const AttendCoefs& cfh,
                                int n_groups, hipStream_t s) {
  constexpr int lds = attend128_lds(KB, VB, VKIND != 0, FUSED);
  static_assert(I8_TABLE_BYTES + lds <= 160 * 1024, "LDS budget");
  static LdsLimit lds_limit;  // per instantiation: the limit is raised once per device
  if (const hipError_t e = raise_lds_limit(lds_limit, reinterpret_cast<const void*>(&attend128_kernel<KB, KPROD, VB, VKIND, FUSED>), lds); e != hipSuccess) return e;
  const dim3 grid(a.nchunks, n_groups, (a.q_per_group + 3) / 4);
  hipLaunchKernelGGL((attend128_kernel<KB, KPROD, VB, VKIND, FUSED>), grid, dim3(512), lds, s, ka, a, cf, cfh);
  return hipGetLastError();
}

// all key variants for one kind of value code; kb < 0: logits from a.scores
template <int VB, int VKIND>
hipError_t launch_attend128_vb(int kb, bool kprod, const ScoreI8Args& ka, const AttendArgs& a, const AttendCoefs& cf,
                               const AttendCoefs& cfh, int n_groups, hipStream_t s) {
  if (kb < 0) return launch_attend128_one<0, false, VB, VKIND, false>(ka, a, cf, cfh, n_groups, s);
  switch (kb * 2 + (kprod ? 1 : 0)) {
    case 1: return launch_attend128_one<0, true, VB, VKIND, true>(ka, a, cf, cfh, n_groups, s);
    case 2: return launch_attend128_one<1, false, VB, VKIND, true>(ka, a, cf, cfh, n_groups, s);
    case 3: return launch_attend128_one<1, true, VB, VKIND, true>(ka, a, cf, cfh, n_groups, s);
    case 4: return launch_attend128_one<2, false, VB, VKIND, true>(ka, a, cf, cfh, n_groups, s);
    case 5: return launch_attend128_one<2, true, VB, VKIND, true>(ka, a, cf, cfh, n_groups, s);
    case 6: return launch_attend128_one<3, false, VB, VKIND, true>(ka, a, cf, cfh, n_groups, s);
    case 7: return launch_attend128_one<3, true, VB, VKIND, true>(ka, a, cf, cfh, n_groups, s);
    case 8: return launch_attend128_one<4, false, VB, VKIND, true>(ka, a, cf, cfh, n_groups, s);
    case 9: return launch_attend128_one<4, true, VB, VKIND, true>(ka, a, cf, cfh, n_groups, s);
    default: return hipErrorInvalidValue;
  }
}

// one translation unit per kind of value code (tq_attend_128_v*.hip: MSE codes of 1..4 bits; tq_attend_128_p*.hip:
// codes of Alg. 2 with 0..2 index bits; tq_attend_128_s*.hip: two instances with 1 + 2 or 2 + 3 index bits: what fits
// LDS beside the second set of weights)
#define TQ_ATTEND128_DECL(NAME)                                                                  \
  hipError_t NAME(int kb, bool kprod, const ScoreI8Args& ka, const AttendArgs& a, const AttendCoefs& cf, \
                  const AttendCoefs& cfh, int n_groups, hipStream_t s)
TQ_ATTEND128_DECL(launch_attend128_v1);
TQ_ATTEND128_DECL(launch_attend128_v2);
TQ_ATTEND128_DECL(launch_attend128_v3);
TQ_ATTEND128_DECL(launch_attend128_v4);
TQ_ATTEND128_DECL(launch_attend128_p0);
TQ_ATTEND128_DECL(launch_attend128_p1);
TQ_ATTEND128_DECL(launch_attend128_p2);
TQ_ATTEND128_DECL(launch_attend128_s1);
TQ_ATTEND128_DECL(launch_attend128_s2);

}  // namespace tq
