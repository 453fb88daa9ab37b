// Scoring for a few queries per code, integer-matrix-core version.
//
// The estimator of Sec. 3.2 in the rotated basis,
//     s = nu * ( sum_j qr_j c[idx_j]  +  kappa gamma sum_j qs_j z_j ),
// only ever multiplies query coordinates by a function of a few BITS of the
// code.  Over the bit planes b_p of idx (the packed layout stores exactly these
// planes) the centroid table has the Walsh expansion
//     c[idx] = sum over subsets S of planes of  w_S * prod_{p in S} (2 b_p - 1),
// and a product of +-1 factors is +-1 according to the parity of the planes in
// S, i.e. to one bit of the XOR of those plane words.  Hence
//     sum_j qr_j c[idx_j] = const * sum_j qr_j + sum_S coef_S * M_S,
//     M_S = sum of qr_j over the coordinates where the XOR of the planes in S is 1,
// and likewise sum_j qs_j z_j = 2 * M_Z - sum_j qs_j with Z the qjl plane.
// A codebook that is symmetric about zero (the Lloyd-Max solution for the
// symmetric coordinate density of Lemma 1 is) has w_S = 0 for every S of even
// size, which leaves 1, 2, 4, 8 terms for 1..4 bits; terms whose coefficient is
// exactly zero are never formed: this path is taken only for tables with
// c[K-1-v] = -c[v] exactly (score_i8_applicable), nothing is approximated.
// Every M is a 0/1-masked sum: an int8 x int8 contraction on the matrix cores
// (v_mfma_i32_16x16x64_i8) between fixed-point digits of the queries and the
// mask expanded to one byte per bit; the expansion is one LDS lookup per 8
// coordinates (byte -> 8 bytes) instead of per-coordinate bit fiddling.
//
// Fixed point: per query, Q_j = round(q_j * 2^e) with |Q_j| < 2^20, written in
// balanced base 128: Q = D0 + 2^7 D1 + 2^14 D2 with digits in [-64, 64] (valid
// signed bytes).  Rows of the A operand: 4 queries x (3 digits + one unused
// row).  Integer arithmetic is exact; the only rounding is that of q to 21 bits
// (relative 2^-20 of the query's largest coordinate), far inside 1e-4.
//
// Operand layout of v_mfma_i32_16x16x64_i8: A row / B column = lane % 16, the
// lane's 16 bytes are 16 values of k for k-chunk lane / 16 (any bijection of k
// works as long as A and B use the same one); D[4*(lane/16) + r][lane % 16] in
// register r.  With row = 4*query + digit a lane ends up holding the three
// digit sums for ONE (query, key) pair.
//
// Which coordinates a lane feeds: d is a multiple of 128 here, so the d/32
// plane-word groups of a key split evenly over the four k-chunks: lane chunk kq
// owns groups kq, kq+4, ...; k-step s = 2i + h uses half h (16 coordinates) of
// its i-th group.  A lane therefore loads whole words of its own groups only:
// no word is fetched twice and the 16 keys x 4 chunks of a tile read one
// contiguous span of the code arrays.
//
// LDS lookups by data-dependent address collide on banks when all lanes share
// one 2 KB table (measured: that was the bound of this kernel).  The table is
// therefore replicated 32 times, copy c = lane % 32 living in banks 2c, 2c+1
// (entry e of copy c at dword 64 e + 2 c): every lookup is conflict free.  The
// 64 KB table is filled while the code words are in flight.
#include <cstring>

#include "tq_score_i8.h"

#include <type_traits>

namespace tq {

typedef float f32x4 __attribute__((ext_vector_type(4)));


// ---------------------------------------------------------------------------
// Query preparation for the int8 path: rotate / sketch one query per workgroup
// (y = W q for W = Pi or S), choose the fixed-point scale, and write the digit
// bytes in the order the scoring kernel's A operand wants them.
// grid (nq, 1 or 2 matrices), 512 threads.  Row j of W is read by the 32 lanes
// of a half-wavefront, 16 bytes each, and reduced across them.
// ---------------------------------------------------------------------------
template <int P>  // P = d / 128: 16-byte pieces per lane per row; a half-wavefront owns 8 P rows
__global__ __launch_bounds__(512) void prep_i8_kernel(const int d, const int d_hi, const float* __restrict__ W0,
                                                      const float* __restrict__ W1,
                                                      const float* __restrict__ x, const int64_t ldx,
                                                      uint4* __restrict__ img, float* __restrict__ scal) {
  __shared__ float ys[512];
  __shared__ float red_mx[8];
  __shared__ int red_tot[8], red_hi[8];
  const int tid = threadIdx.x;
  const int l32 = tid & 31, hw = tid >> 5;  // 16 half-wavefronts
  const int64_t q = blockIdx.x;
  const int mat = blockIdx.y;
  const float* W = mat == 0 ? W0 : W1;
  // this lane's share of the query, then 8 rows at a time, all their loads in flight together
  f32x4 xv[P];
#pragma unroll
  for (int c = 0; c < P; ++c) xv[c] = *reinterpret_cast<const f32x4*>(x + q * ldx + 128 * c + 4 * l32);
#pragma unroll 1
  for (int r0 = 0; r0 < 8 * P; r0 += 8) {
    f32x4 wv[8][P];
#pragma unroll
    for (int r = 0; r < 8; ++r)
#pragma unroll
      for (int c = 0; c < P; ++c)
        wv[r][c] = *reinterpret_cast<const f32x4*>(W + (int64_t)(hw + 16 * (r0 + r)) * d + 128 * c + 4 * l32);
    float part[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      float acc = 0.f;
#pragma unroll
      for (int c = 0; c < P; ++c) {
        acc = fmaf(wv[r][c].x, xv[c].x, acc); acc = fmaf(wv[r][c].y, xv[c].y, acc);
        acc = fmaf(wv[r][c].z, xv[c].z, acc); acc = fmaf(wv[r][c].w, xv[c].w, acc);
      }
      part[r] = acc;
    }
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1)
#pragma unroll
      for (int r = 0; r < 8; ++r) part[r] += __shfl_xor(part[r], off);
#pragma unroll
    for (int r = 0; r < 8; ++r)
      if (l32 == r) ys[hw + 16 * (r0 + r)] = part[r];
  }
  __syncthreads();
  float mx = tid < d ? fabsf(ys[tid]) : 0.f;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  if ((tid & 63) == 0) red_mx[tid >> 6] = mx;
  __syncthreads();
  mx = red_mx[0];
#pragma unroll
  for (int w = 1; w < 8; ++w) mx = fmaxf(mx, red_mx[w]);
  // power-of-two scale with |Q| < 2^20
  int e = 0;
  if (mx > 0.f) (void)frexpf(mx, &e);  // mx = f * 2^e, f in [0.5, 1)
  const float sc = ldexpf(1.f, 19 - e);
  int tot = tid < d ? __float2int_rn(ys[tid] * sc) : 0;
  int tot_hi = tid < d_hi ? tot : 0;  // the first d_hi coordinates: instance hi of a split (Sec. 4.3)
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    tot += __shfl_xor(tot, off);
    tot_hi += __shfl_xor(tot_hi, off);
  }
  if ((tid & 63) == 0) {
    red_tot[tid >> 6] = tot;
    red_hi[tid >> 6] = tot_hi;
  }
  __syncthreads();
  if (tid == 0) {
    int t = 0, th = 0;
#pragma unroll
    for (int w = 0; w < 8; ++w) {
      t += red_tot[w];
      th += red_hi[w];
    }
    scal[(q * 2 + mat) * 4 + 0] = ldexpf(1.f, e - 19);
    scal[(q * 2 + mat) * 4 + 1] = (float)t * ldexpf(1.f, e - 19);
    scal[(q * 2 + mat) * 4 + 2] = (float)th * ldexpf(1.f, e - 19);
    scal[(q * 2 + mat) * 4 + 3] = (float)(t - th) * ldexpf(1.f, e - 19);
  }
  const int ks = d >> 6;
  for (int u = tid; u < ks * 16; u += 512) {  // unit = (k-step s, digit dg, k-chunk kq)
    const int kq = u & 3, dg = (u >> 2) & 3, s = u >> 4;
    const int c0 = i8_coord0(s, kq);
    uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      // balanced digits: D0, D1 in [-64, 63], D2 in [-64, 64]
      const int Q = __float2int_rn(ys[c0 + k] * sc);
      const int d0 = ((Q + 64) & 127) - 64;
      const int Q1 = (Q - d0) >> 7;
      const int d1 = ((Q1 + 64) & 127) - 64;
      const int d2 = (Q1 - d1) >> 7;
      const int dig = dg == 0 ? d0 : dg == 1 ? d1 : dg == 2 ? d2 : 0;
      w[k >> 2] |= ((uint32_t)dig & 0xFFu) << (8 * (k & 3));
    }
    img[((q * 2 + mat) * ks + s) * 16 + dg * 4 + kq] = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// The same images for vectors of more than 512 coordinates, from queries that a matrix-vector kernel has already
// rotated (y0 = Pi q, y1 = S q, [nq][d] fp32): scale, sums and digit bytes as prep_i8_kernel writes them.
// grid (nq, 1 or 2), 512 threads.
__global__ __launch_bounds__(512) void digitise_i8_kernel(const int d, const float* __restrict__ y0,
                                                          const float* __restrict__ y1, uint4* __restrict__ img,
                                                          float* __restrict__ scal) {
  __shared__ float red_mx[8];
  __shared__ long long red_tot[8];
  const int tid = threadIdx.x;
  const int64_t q = blockIdx.x;
  const int mat = blockIdx.y;
  const float* const y = (mat == 0 ? y0 : y1) + q * d;
  float mx = 0.f;
  for (int k = tid; k < d; k += 512) mx = fmaxf(mx, fabsf(y[k]));
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  if ((tid & 63) == 0) red_mx[tid >> 6] = mx;
  __syncthreads();
  mx = red_mx[0];
#pragma unroll
  for (int w = 1; w < 8; ++w) mx = fmaxf(mx, red_mx[w]);
  int e = 0;
  if (mx > 0.f) (void)frexpf(mx, &e);  // mx = f * 2^e, f in [0.5, 1): |Q| < 2^20 below
  const float sc = ldexpf(1.f, 19 - e);
  long long tot = 0;  // up to 4096 values below 2^20
  for (int k = tid; k < d; k += 512) tot += __float2int_rn(y[k] * sc);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) tot += __shfl_xor(tot, off);
  if ((tid & 63) == 0) red_tot[tid >> 6] = tot;
  __syncthreads();
  if (tid == 0) {
    long long t = 0;
#pragma unroll
    for (int w = 0; w < 8; ++w) t += red_tot[w];
    scal[(q * 2 + mat) * 4 + 0] = ldexpf(1.f, e - 19);
    scal[(q * 2 + mat) * 4 + 1] = (float)t * ldexpf(1.f, e - 19);
    scal[(q * 2 + mat) * 4 + 2] = 0.f;  // one instance
    scal[(q * 2 + mat) * 4 + 3] = (float)t * ldexpf(1.f, e - 19);
  }
  const int ks = d >> 6;
  for (int u = tid; u < ks * 16; u += 512) {  // unit = (k-step s, digit dg, k-chunk kq)
    const int kq = u & 3, dg = (u >> 2) & 3, s = u >> 4;
    const int c0 = i8_coord0(s, kq);
    uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      const int Q = __float2int_rn(y[c0 + k] * sc);
      const int d0 = ((Q + 64) & 127) - 64;
      const int Q1 = (Q - d0) >> 7;
      const int d1 = ((Q1 + 64) & 127) - 64;
      const int d2 = (Q1 - d1) >> 7;
      const int dig = dg == 0 ? d0 : dg == 1 ? d1 : dg == 2 ? d2 : 0;
      w[k >> 2] |= ((uint32_t)dig & 0xFFu) << (8 * (k & 3));
    }
    img[((q * 2 + mat) * ks + s) * 16 + dg * 4 + kq] = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// KSM: compile-time bound on the number of 64-coordinate k-steps (register arrays).
// A wavefront owns i8_tiles() tiles of 16 keys and requests all their code words up front.
// WALK: the grid is sized to the chip and a workgroup walks several blocks of keys (see launch_one).
template <int BITS, bool PROD, int KSM, bool WALK = (BITS < 4)>
__global__ __launch_bounds__(512) void score_i8_kernel(const ScoreI8Args a) {
  __shared__ __attribute__((aligned(16))) uint2 expand_s[256 * I8_COPIES];  // [256][32]: byte -> one byte per bit
  constexpr int GI = KSM / 2;      // plane-word groups per lane
  constexpr int TILES = i8_tiles(BITS, KSM);  // tiles per wavefront
  constexpr int NM = (1 << BITS) - 1;
  constexpr int NW = BITS > 0 ? BITS : 1;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // in a scalar register: addresses built from it are uniform
  const int col = lane & 15;   // key within a tile / row of A
  const int kq = lane >> 4;    // k-chunk; also the query whose sums this lane receives
  const int group = blockIdx.y;
  const int q0 = blockIdx.z * 4;
  const int d = a.d;
  const int ks_all = d >> 6;   // k-steps of 64 coordinates of the whole vector (even): the stride of the images
  const int ks = a.ks_slice;   // k-steps of this launch (even, at most KSM), starting at a.k0
  const int gi = ks >> 1;

  // lane = row + 16*kq of the A operand, row = 4*query + digit
  const int a_query = col >> 2, a_digit = col & 3;
  const bool a_live = q0 + a_query < a.q_per_group;
  const int64_t qrow = (int64_t)group * a.q_per_group + q0 + (a_live ? a_query : 0);
  // the query kq whose results this lane receives
  const bool out_live = q0 + kq < a.q_per_group;
  const int64_t orow = (int64_t)group * a.q_per_group + q0 + (out_live ? kq : 0);
  v4i ar[KSM], as_[KSM];
  float r_inv = 0.f, r_sum = 0.f, s_inv = 0.f, s_sum = 0.f;

  // ---- 1. A operands first (loads return in order): digit images and scalars written by
  // prep_i8_kernel ------------------------------------------------------------------------
#pragma unroll
  for (int s = 0; s < KSM; ++s) {
    uint4 r = make_uint4(0, 0, 0, 0), z = make_uint4(0, 0, 0, 0);
    if (s < ks) {
      if (BITS > 0) r = a.img[((qrow * 2 + 0) * ks_all + a.k0 + s) * 16 + a_digit * 4 + kq];
      if (PROD) z = a.img[((qrow * 2 + 1) * ks_all + a.k0 + s) * 16 + a_digit * 4 + kq];
    }
    ar[s] = v4i{(int)r.x, (int)r.y, (int)r.z, (int)r.w};
    as_[s] = v4i{(int)z.x, (int)z.y, (int)z.z, (int)z.w};
  }
  if (BITS > 0) {
    r_inv = a.scal[(orow * 2 + 0) * 4];
    r_sum = a.scal[(orow * 2 + 0) * 4 + 1];
  }
  if (PROD) {
    s_inv = a.scal[(orow * 2 + 1) * 4];
    s_sum = a.scal[(orow * 2 + 1) * 4 + 1];
  }

  // ---- 2. every code word of this wavefront's keys goes in flight: the first tile can start
  // while the later ones are still on their way ------------------------------------------
  const int groups = d >> 5;
  const int words_per_row = groups * BITS;
  const int64_t gbase = (int64_t)group * a.n;
  // A workgroup walks blocks of 8 x 16 TILES keys (the grid may be sized to the chip instead of to the keys): the
  // table and the query operands are set up once per workgroup.  The first block's code words are requested
  // before the table is filled, so that the fill runs while they are on their way.
  const int64_t nblk = (a.n + 8 * 16 * TILES - 1) / (8 * 16 * TILES);
  int64_t blk = blockIdx.x;  // below nblk: the grid has at most that many workgroups along x
  int64_t wave_key0 = (blk * 8 + wave) * (16 * TILES);
  bool full = wave_key0 + 16 * TILES <= a.n;  // uniform: no key of this wavefront is past the end
  uint32_t pw[TILES][GI][NW], zw[TILES][GI];
  float kg[TILES], nu[TILES];
  auto load_codes = [&](auto clamp_c) {
    constexpr bool CLAMP = decltype(clamp_c)::value;
    // one base address per array and lane; without clamping the tiles are constant offsets from it
    const int64_t key0 = wave_key0 + col;
    const int64_t row0 = gbase + (key0 < a.n ? key0 : a.n - 1);
    const int g0 = 2 * a.k0;  // first plane-word group of this launch (a k-step is two groups)
    const uint32_t* const pi0 = a.idx + row0 * words_per_row + (g0 + kq) * BITS;
    const uint32_t* const pz0 = a.qjl + (PROD ? row0 * groups + g0 + kq : 0);
    const float* const pg0 = a.gamma + (PROD ? row0 : 0);
    const float* const pn0 = a.norm + (a.norm != nullptr ? row0 : 0);
#pragma unroll
    for (int t = 0; t < TILES; ++t) {
      // rows advance by 16 per tile; a clamped row (results of such lanes are not stored) moves
      // back by the same number of rows in every array
      int back = 0;
      if (CLAMP) back = (int)(key0 + 16 * t < a.n ? 0 : key0 + 16 * t - (a.n - 1)) - (int)(key0 < a.n ? 0 : key0 - (a.n - 1));
      const int dr = 16 * t - back;  // row - row0
      const uint32_t* pi = pi0 + dr * words_per_row;
      const uint32_t* pz = pz0 + dr * groups;
#pragma unroll
      for (int i = 0; i < GI; ++i) {
        const int io = i < gi ? i : 0;
#pragma unroll
        for (int pl = 0; pl < BITS; ++pl) pw[t][i][pl] = pi[io * 4 * BITS + pl];
        zw[t][i] = PROD ? pz[io * 4] : 0u;
      }
      kg[t] = PROD ? pg0[dr] : 0.f;
      nu[t] = a.norm != nullptr ? pn0[dr] : 1.f;
    }
  };
  if (full) load_codes(std::false_type{});
  else load_codes(std::true_type{});

  // ---- 3. the expansion table, 32 bank-private copies ------------------------------------
  // thread -> (entry tid/32 + 16 i, copy tid%32): consecutive threads write consecutive
  // addresses; the low nibble of the entry is the thread's own, the high nibble is i
  {
    const uint32_t lo = (((uint32_t)tid >> 5) * 0x00204081u) & 0x01010101u;  // bit i of the nibble -> byte i
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const uint32_t hi = ((uint32_t)i * 0x00204081u) & 0x01010101u;
      expand_s[tid + 512 * i] = make_uint2(lo, hi);
    }
  }
  __syncthreads();

  const uint32_t copy_off = (uint32_t)(lane & (I8_COPIES - 1)) * 8u;
  const char* const table = reinterpret_cast<const char*>(expand_s);
  // bits [16 h, 16 h + 16) of w -> 16 bytes of 0/1.  Table offset = 256 * byte + 8 * copy: one
  // byte permute puts byte k of w into bits 8..15 above the copy offset in bits 0..7.
  auto expand16 = [&](uint32_t w, int h) -> v4i {
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
  float cr[NM > 0 ? NM : 1];
#pragma unroll
  for (int m = 1; m <= NM; ++m) cr[m - 1] = a.coef[m] * r_inv;
  const bool add = a.accumulate != 0;  // uniform: the code-independent terms came with an earlier launch
  const float base_r = add ? 0.f : a.coef[0] * r_sum;
  const float zs = 2.f * s_inv;
  if (add) s_sum = 0.f;
  float* out0 = a.scores + ((int64_t)group * a.q_per_group + q0 + kq) * a.lds + wave_key0 + col;

  // The tiles run as a three-stage software pipeline, written out in source order: while the
  // MFMAs of tile t issue, the table lookups of tile t+1 are already on their way and the
  // sums of tile t-1 are combined and stored, so no stage waits for its own latency.
  // A wavefront whose keys all exist runs it without per-tile bounds tests; the last
  // wavefront of a group takes the guarded version.
  constexpr int NT = (BITS > 0 ? (1 << (BITS - 1)) : 0) + (PROD ? 1 : 0);  // masked sums per tile
  constexpr int NTA = NT > 0 ? NT : 1;
  auto run_tiles = [&](auto full_c) {
    constexpr bool FULL = decltype(full_c)::value;
    constexpr bool PIPE = KSM * NTA <= 12;
    v4i bop[2][PIPE ? KSM : 1][NTA];  // expanded B operands of the tiles in flight
    v4i acc[2][NTA];       // sums of two tiles
    auto lookups = [&](int t, v4i (&b)[PIPE ? KSM : 1][NTA]) {
      if (!PIPE) return;
#pragma unroll
      for (int s = 0; s < KSM; ++s) {
        if (s >= ks) break;
        int j = 0;
#pragma unroll
        for (int m = 1; m <= NM; ++m) {
          if (!i8_term(m)) continue;
          uint32_t w = 0u;
#pragma unroll
          for (int pl = 0; pl < BITS; ++pl)
            if (m & (1 << pl)) w ^= pw[t][s >> 1][pl];
          b[s][j++] = expand16(w, s & 1);
        }
        if (PROD) b[s][j] = expand16(zw[t][s >> 1], s & 1);
      }
    };
    auto mfmas = [&](const v4i (&b)[PIPE ? KSM : 1][NTA], v4i (&c)[NTA]) {
      if (!PIPE) return;
#pragma unroll
      for (int j = 0; j < NTA; ++j) c[j] = v4i{0, 0, 0, 0};
#pragma unroll
      for (int s = 0; s < KSM; ++s) {  // unrolled so the A registers are indexed statically
        if (s >= ks) break;
#pragma unroll
        for (int j = 0; j < NT; ++j)
          c[j] = __builtin_amdgcn_mfma_i32_16x16x64_i8((PROD && j == NT - 1) ? as_[s] : ar[s], b[s][j], c[j], 0, 0, 0);
      }
    };
    auto finish = [&](int t, const v4i (&c)[NTA]) {
      float total = base_r;
      int j = 0;
#pragma unroll
      for (int m = 1; m <= NM; ++m)
        if (i8_term(m)) total = fmaf(cr[m - 1], digits_sum(c[j++]), total);
      if (PROD) total = fmaf(a.kappa * kg[t], fmaf(zs, digits_sum(c[NT - 1]), -s_sum), total);
      total *= nu[t];
      if (out_live && (FULL || wave_key0 + t * 16 + col < a.n)) out0[t * 16] = add ? out0[t * 16] + total : total;
    };
    if (PIPE) {
      lookups(0, bop[0]);
#pragma unroll
      for (int t = 0; t < TILES; ++t) {
        if (!FULL && wave_key0 + t * 16 >= a.n) {  // uniform over the wavefront
          if (t > 0) finish(t - 1, acc[(t - 1) & 1]);
          return;
        }
        if (t + 1 < TILES) lookups(t + 1, bop[(t + 1) & 1]);
        mfmas(bop[t & 1], acc[t & 1]);
        if (t > 0) finish(t - 1, acc[(t - 1) & 1]);
      }
      finish(TILES - 1, acc[(TILES - 1) & 1]);
    } else {
      // too many operand registers for two tiles in flight: one k-step of one tile at a time
#pragma unroll
      for (int t = 0; t < TILES; ++t) {
        if (!FULL && wave_key0 + t * 16 >= a.n) return;
#pragma unroll
        for (int j = 0; j < NTA; ++j) acc[0][j] = v4i{0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < KSM; ++s) {
          if (s >= ks) break;
          int j = 0;
#pragma unroll
          for (int m = 1; m <= NM; ++m) {
            if (!i8_term(m)) continue;
            uint32_t w = 0u;
#pragma unroll
            for (int pl = 0; pl < BITS; ++pl)
              if (m & (1 << pl)) w ^= pw[t][s >> 1][pl];
            acc[0][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ar[s], expand16(w, s & 1), acc[0][j], 0, 0, 0);
            ++j;
          }
          if (PROD)
            acc[0][NT - 1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(as_[s], expand16(zw[t][s >> 1], s & 1), acc[0][NT - 1], 0, 0, 0);
        }
        finish(t, acc[0]);
      }
    }
  };
  while (true) {
    if (full) run_tiles(std::true_type{});
    else run_tiles(std::false_type{});
    if constexpr (!WALK) break;  // a workgroup per block of keys: straight-line code
    blk += gridDim.x;
    if (blk >= nblk) break;  // uniform over the workgroup
    wave_key0 = (blk * 8 + wave) * (16 * TILES);
    full = wave_key0 + 16 * TILES <= a.n;
    out0 = a.scores + ((int64_t)group * a.q_per_group + q0 + kq) * a.lds + wave_key0 + col;
    if (full) load_codes(std::false_type{});
    else load_codes(std::true_type{});
  }
}

template <int BITS, bool PROD, int KSM>
static hipError_t launch_one(const ScoreI8Args& a, int n_groups, hipStream_t s) {
  const int64_t per_wg = 8 * 16 * i8_tiles(BITS, KSM);
  // two workgroups fit a compute unit (64 KB of LDS each): about that many in all, each walking its share of the
  // keys.  Up to 3 index bits, that is: the 4-bit kernel, with half the keys per block, loses more to the loads of
  // a block waiting for the block before it than it gains (d = 1536, 10^6 codes: 92 against 84 us per launch; 1 + 1
  // bits at d = 3072: 86 against 110), so there every block of keys gets a workgroup of its own.
  const int64_t others = (int64_t)n_groups * ((a.q_per_group + 3) / 4);
  const int64_t nblk = (a.n + per_wg - 1) / per_wg;
  int64_t gx = BITS >= 4 ? nblk : (2 * (int64_t)device_cu_count() + others - 1) / others;
  if (gx > nblk) gx = nblk;
  if (gx < 1) gx = 1;
  const dim3 grid((unsigned)gx, n_groups, (a.q_per_group + 3) / 4);
  hipLaunchKernelGGL((score_i8_kernel<BITS, PROD, KSM>), grid, dim3(512), 0, s, a);
  return hipGetLastError();
}

template <int BITS, bool PROD>
static hipError_t launch_ks(const ScoreI8Args& a, int n_groups, hipStream_t s) {
  const int ks = a.ks_slice;
  if (ks <= 2) return launch_one<BITS, PROD, 2>(a, n_groups, s);
  if (ks <= 4) return launch_one<BITS, PROD, 4>(a, n_groups, s);
  return launch_one<BITS, PROD, 8>(a, n_groups, s);
}

template <int BITS>
static hipError_t launch_bits(const ScoreI8Args& a, bool prod, int n_groups, hipStream_t s) {
  return prod ? launch_ks<BITS, true>(a, n_groups, s) : launch_ks<BITS, false>(a, n_groups, s);
}

// digit images and scalars of nq queries; beyond 512 coordinates also the rotated / sketched queries in fp32,
// which a kernel of their own digitises
size_t score_i8_workspace_bytes(int d, int64_t nq) {
  const size_t images = (size_t)nq * 2 * ((size_t)(d >> 6) * 256 + 16) + 512;
  return d > 64 * I8_MAX_KS ? images + 2 * ((size_t)nq * d * sizeof(float) + 256) : images;
}

// Walsh coefficients of the centroid table over the bit planes of the index:
//   c[v] = sum_S w_S chi_S(v),  chi_S(v) = prod_{p in S} (2 v_p - 1) = sgn_S * (2 x_S(v) - 1),
// x_S(v) = XOR of the bits of v in S, sgn_S = +1 for odd |S| and -1 for even |S|.  Summed in
// pairs (v, K-1-v): for even |S| chi_S agrees on the pair, so a table with c[K-1-v] = -c[v]
// gives exactly zero there.
void i8_walsh(int bits, const Codebook& cb, double* w) {
  const int K = 1 << bits;
  for (int sset = 0; sset < K; ++sset) {
    double acc = 0.0;
    const int size = __builtin_popcount(sset);
    for (int v = 0; v < (K > 1 ? K / 2 : 1); ++v) {
      const int par = __builtin_popcount(v & sset) & 1;
      const double chi = ((size - par) & 1) ? -1.0 : 1.0;  // (-1)^(number of zero bits of v in S)
      if (K == 1) acc += cb.c[0];
      else if (size & 1) acc += chi * ((double)cb.c[v] - (double)cb.c[K - 1 - v]);
      else acc += chi * ((double)cb.c[v] + (double)cb.c[K - 1 - v]);
    }
    w[sset] = acc / K;
  }
}

// the d = 128 preparation kernel for the split variant (tq_score_i8_split.hip)
hipError_t launch_prep_i8_128(int d_hi, const float* Pi, const float* S, const float* q, int64_t ldq, int64_t nq,
                              bool prod, uint4* img, float* scal, hipStream_t stream) {
  hipLaunchKernelGGL(prep_i8_kernel<1>, dim3((unsigned)nq, prod ? 2 : 1), dim3(512), 0, stream, 128, d_hi, Pi, S, q, ldq,
                     img, scal);
  return hipGetLastError();
}

// sum_j q_j c[idx_j] = coef[0] * sum_j q_j + sum over the odd-sized plane subsets S of coef[S] * M_S, where M_S
// is the sum of q_j over the coordinates whose index bits in S XOR to 1.  False for a table that is not
// symmetric about zero (its even-sized subsets do not vanish).
bool i8_coefficients(int bits, const Codebook& cb, float* coef) {
  double w[16];
  i8_walsh(bits, cb, w);
  const int K = 1 << bits;
  double c0 = w[0];
  for (int v = 0; v < 16; ++v) coef[v] = 0.f;
  for (int sset = 1; sset < K; ++sset) {
    const double sgn = (__builtin_popcount(sset) & 1) ? 1.0 : -1.0;
    if (!i8_term(sset) && w[sset] != 0.0) return false;
    c0 -= sgn * w[sset];
    coef[sset] = (float)(2.0 * sgn * w[sset]);
  }
  coef[0] = (float)c0;
  return true;
}

bool score_i8_applicable(int bits, int d, const Codebook& cb) {
  if (bits < 0 || bits > 4 || d % 128 != 0 || d > I8_MAX_D) return false;
  double w[16];
  i8_walsh(bits, cb, w);
  for (int sset = 1; sset < (1 << bits); ++sset)
    if (!i8_term(sset) && w[sset] != 0.0) return false;  // not symmetric about zero
  return true;
}

// Arguments of the single-kernel d = 128 path (tq_score_i8_128_body.h) for callers that run it inside a
// kernel of their own; false when that path does not take these codes.
bool score128_args(int bits, bool prod, const float* PiT, const float* ST, const float* q, int64_t ldq,
                   const uint32_t* idx, const uint32_t* qjl, const float* gamma, const float* norm, int64_t n,
                   int n_groups, int q_per_group, float kappa, const Codebook& cb, int64_t group_stride, ScoreI8Args* a) {
  const auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
  if (bits < 0 || bits > 4 || !(bits > 0 || prod)) return false;
  if (bits > 0 && (PiT == nullptr || idx == nullptr || !al16(idx))) return false;
  if (prod && (ST == nullptr || qjl == nullptr || gamma == nullptr || !al16(qjl))) return false;
  std::memset(a, 0, sizeof(*a));
  a->PiT = PiT; a->ST = ST; a->x = q; a->ldx = ldq; a->idx = idx; a->qjl = qjl; a->gamma = gamma; a->norm = norm;
  a->n = n; a->group_stride = group_stride; a->total_rows = (int64_t)(n_groups - 1) * group_stride + n; a->d = 128; a->q_per_group = q_per_group; a->kappa = kappa;
  return i8_coefficients(bits, cb, a->coef);
}

hipError_t launch_score_i8(int bits, bool prod, const float* Pi, const float* S, const float* PiT, const float* ST,
                           const float* q, int64_t ldq,
                           void* workspace, const uint32_t* idx, const uint32_t* qjl, const float* gamma,
                           const float* norm, float* scores, int64_t lds, int64_t n, int d, int n_groups,
                           int q_per_group, float kappa, const Codebook& cb, hipStream_t stream) {
  if (n_groups == 0 || q_per_group == 0) return hipSuccess;
  if (bits < 0 || bits > 4 || d % 128 != 0 || d > I8_MAX_D) return hipErrorInvalidValue;
  const int64_t nq = (int64_t)n_groups * q_per_group;
  uint4* img = static_cast<uint4*>(workspace);
  float* scal = reinterpret_cast<float*>(static_cast<char*>(workspace) + (size_t)nq * 2 * (d >> 6) * 256);
  if (n == 0) return hipSuccess;
  ScoreI8Args a;
  a.img = img; a.scal = scal; a.PiT = PiT; a.ST = ST; a.x = q; a.ldx = ldq; a.idx = idx; a.qjl = qjl; a.gamma = gamma; a.norm = norm;
  a.scores = scores; a.lds = lds; a.n = n; a.total_rows = (int64_t)n_groups * n; a.group_stride = n; a.d = d; a.q_per_group = q_per_group; a.kappa = kappa;
  a.k0 = 0; a.ks_slice = d >> 6; a.accumulate = 0;
  if (!i8_coefficients(bits, cb, a.coef)) return hipErrorInvalidValue;  // see score_i8_applicable
  // d = 128 with the transposed matrices at hand and 16-byte aligned codes: one kernel does it all
  const auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
  if (d == 128 && (bits > 0 || prod) && (bits == 0 || (PiT != nullptr && al16(idx))) &&
      (!prod || (ST != nullptr && al16(qjl))))
    return launch_score_i8_128(bits, prod, a, n_groups, stream);
  const dim3 pgrid((unsigned)nq, prod ? 2 : 1);
  if (d > 64 * I8_MAX_KS) {
    // long vectors: the matrix-vector kernel rotates the queries into the workspace, then their digits are written
    const size_t images = ((size_t)nq * 2 * ((size_t)(d >> 6) * 256 + 16) + 512 + 255) / 256 * 256;
    float* const qr = reinterpret_cast<float*>(static_cast<char*>(workspace) + images);
    float* const qs = reinterpret_cast<float*>(static_cast<char*>(workspace) + images + ((size_t)nq * d * sizeof(float) + 255) / 256 * 256);
    if (const hipError_t e = launch_matvec_small(d, (int)nq, Pi, prod ? S : nullptr, q, ldq, qr, qs, stream); e != hipSuccess) return e;
    hipLaunchKernelGGL(digitise_i8_kernel, pgrid, dim3(512), 0, stream, d, qr, qs, img, scal);
  } else {
    switch (d >> 7) {
      case 1: hipLaunchKernelGGL(prep_i8_kernel<1>, pgrid, dim3(512), 0, stream, d, 0, Pi, S, q, ldq, img, scal); break;
      case 2: hipLaunchKernelGGL(prep_i8_kernel<2>, pgrid, dim3(512), 0, stream, d, 0, Pi, S, q, ldq, img, scal); break;
      case 3: hipLaunchKernelGGL(prep_i8_kernel<3>, pgrid, dim3(512), 0, stream, d, 0, Pi, S, q, ldq, img, scal); break;
      default: hipLaunchKernelGGL(prep_i8_kernel<4>, pgrid, dim3(512), 0, stream, d, 0, Pi, S, q, ldq, img, scal); break;
    }
  }
  if (const hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  // 512 coordinates per launch; the launches after the first add to the scores
  const int ks_all = d >> 6;
  for (int k0 = 0; k0 < ks_all; k0 += I8_MAX_KS) {
    a.k0 = k0;
    a.ks_slice = ks_all - k0 < I8_MAX_KS ? ks_all - k0 : I8_MAX_KS;
    a.accumulate = k0 > 0;
    hipError_t e;
    switch (bits) {
      case 0: e = launch_bits<0>(a, prod, n_groups, stream); break;
      case 1: e = launch_bits<1>(a, prod, n_groups, stream); break;
      case 2: e = launch_bits<2>(a, prod, n_groups, stream); break;
      case 3: e = launch_bits<3>(a, prod, n_groups, stream); break;
      case 4: e = launch_bits<4>(a, prod, n_groups, stream); break;
      default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace tq
