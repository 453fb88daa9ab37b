// Few queries per code at d = 128 (attention logits against a quantised key
// cache, Sec. 4.3): one kernel does everything.  The arithmetic is that of
// tq_score_i8.hip (masked sums of fixed-point query digits on
// v_mfma_i32_16x16x64_i8, Walsh terms of a symmetric codebook); what differs is
// how the data gets to the matrix cores.
//
// Measured with cycle stamps inside the kernel: what a workgroup waits for is
// not the MFMAs but its own loads.  When every compute unit asks for its 240 KB
// at once they arrive over about 17 000 cycles (the chip's HBM rate shared by
// 256 workgroups: 10-14 bytes per clock each), and a lane that fetches its own
// 8-byte share of 16 different code rows makes the memory pipeline touch every
// cache line four times on top of that.  So here
//   * a wavefront reads the codes of its keys as plain contiguous 16-byte-per-
//     lane loads (1 KB per instruction) and parks them in a private LDS region;
//     the tiles later pick their words out of LDS in operand order,
//   * the workgroup prepares its own four queries while those loads are in
//     flight (y = Pi q and S q from the transposed matrices, column per thread,
//     query coordinates through scalar registers; then digits into LDS).  That
//     re-reads 128 KB of matrices per workgroup, which is cheaper than the
//     launch-and-latency chain of a preparation kernel in front,
//   * the mask operands need no lookup: a stored word ANDed with 0x01010101 << k is already four
//     operand bytes (bit k + 8 b of the word in byte b, worth 2^k), and the query digits are
//     written pre-scaled by 2^(7 - k) to match (I8Prep::digitise<true>), so a tile's operands cost
//     eight ANDs per stored word where a table in LDS cost four 8-byte reads per word and bounded
//     the tile phase (8 x 65536 keys, 4 queries each: 3.4 of 14.3 us).
//
// Workgroup = 512 threads = 8 wavefronts; a wavefront owns 256 consecutive keys
// = 16 tiles of 16, staged ROUND tiles at a time.  grid = (ceil(n / 2048),
// groups, ceil(queries per group / 4)).
#pragma once
#include "tq_score_i8_prep.h"

#include <type_traits>

namespace tq {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// The codes of a wavefront are asked for a few rounds ahead of their use rather than all at once: rounds of 4 tiles
// (64 keys, 3.5 KB at 2 + 1 bits), two in flight.  8 x 65536 keys, 4 queries each, same box: 12.8 us against 13.4
// with everything requested up front (rounds of 8 tiles: 13.4; rounds of 4, three in flight: 13.4; rounds of 8,
// one in flight: 13.1; on another box 12.5 against rounds of 2 tiles with 2 / 3 / 4 / 6 in flight: 13.0 / 12.7 /
// 12.9 / 13.7, and rounds of one tile with 5 / 8 in flight: 13.7 / 14.3).
constexpr int SCORE128_ROUND_TILES = 4, SCORE128_ROUNDS_AHEAD = 2;
constexpr int TILES_128 = 16;  // tiles per wavefront (the default; 8 or 4 where that would leave compute units idle)
// tiles staged in LDS at a time
__host__ __device__ constexpr int round_tiles(int bits) { return bits <= 3 ? 8 : 4; }
// bytes of one wavefront's staging region: idx, qjl, gamma, norm of 16 * round_tiles rows
__host__ __device__ constexpr int stage_bytes(int bits) { return 16 * round_tiles(bits) * (16 * bits + 16 + 4 + 4); }

// staging regions, partial sums of the query preparation (8 KB), one 2 KB digit image per masked sum, scalars
__host__ __device__ constexpr int score128_lds(int bits) { return 8 * stage_bytes(bits) + 2 * 2 * 4 * 128 * 4 + i8_terms(bits, true) * 2048 + 2 * 4 * 4 * 4; }

// The whole kernel as a function of where a finished score goes: sink(t, score, key_live) is
// called once per tile t (TILES tiles of 16 keys per wavefront) by every lane with the score of
// (query q0 + lane / 16, key wave_key0 + 16 t + lane % 16), wave_key0 = (8 blockIdx.x + wave) * 16 TILES.
// dyn_s: score128_lds(BITS) bytes, 8 staging regions, then the query preparation.  All of LDS may be reused after the workgroup's
// next barrier.
template <int BITS, bool PROD, int TILES = TILES_128, int RTP = 0, int INFLIGHT = 0, class Sink>
__device__ __forceinline__ void score128_body(const ScoreI8Args& a, unsigned char* dyn_s, Sink& sink) {
  constexpr int RT0 = RTP > 0 ? RTP : round_tiles(BITS);
  constexpr int RT = RT0 < TILES ? RT0 : TILES;
  constexpr int ROWS = 16 * RT;               // rows staged per round
  constexpr int ROUNDS = TILES / RT;
  constexpr int NM = (1 << BITS) - 1;
  constexpr int NW = BITS > 0 ? BITS : 1;
  // loads per round; where a round's share of an array is not a whole number of them, the lanes past its end
  // repeat its last piece (same address, same value, in memory and in LDS)
  constexpr int PI = ROWS * BITS;                  // 16-byte pieces of plane words per round
  constexpr int NI = (PI + 63) / 64;               // 1 KB loads per round: plane words
  constexpr int NQ = PROD ? (ROWS + 63) / 64 : 0;  // sign words, a 16-byte piece per row
  constexpr int NR = (ROWS + 63) / 64;             // row-per-lane loads per round: gamma, norm
  constexpr int IDX_OFF = 0, QJL_OFF = ROWS * 16 * BITS, GAM_OFF = QJL_OFF + ROWS * 16, NRM_OFF = GAM_OFF + ROWS * 4;
  constexpr int NT = (BITS > 0 ? (1 << (BITS > 0 ? BITS - 1 : 0)) : 0) + (PROD ? 1 : 0);  // masked sums per tile
  constexpr int NTA = NT > 0 ? NT : 1;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // in a scalar register: addresses built from it are uniform
  const int col = lane & 15;   // key within a tile / row of A
  const int kq = lane >> 4;    // k-chunk = plane-word group; also the query whose sums this lane receives
  const int group = blockIdx.y;
  const int q0 = blockIdx.z * 4;

  unsigned char* const stage = dyn_s + wave * stage_bytes(BITS);
  float* const part_s = reinterpret_cast<float*>(dyn_s + 8 * stage_bytes(BITS));        // [2][2][4][128]
  signed char* const dig_s = reinterpret_cast<signed char*>(part_s + 2 * 2 * 4 * 128);  // [term][4][4][128]
  float* const scal_s = reinterpret_cast<float*>(dig_s + i8_terms(BITS, true) * 2048);  // [2][4][4]

  // ---- 1. this thread's column of the transposed matrix: 64 values of k ---------------------
  I8Prep<(BITS > 0), PROD> prep;
  prep.load(a, wave, tid);

  // ---- 2. the codes of this wavefront's keys, as contiguous 16-byte pieces ---------------------
  // Pieces past the end of the arrays are clamped onto the last one (never used: the
  // scores of keys past the end are not stored).
  const int64_t gbase = (int64_t)group * a.group_stride;
  const int64_t wave_key0 = ((int64_t)blockIdx.x * 8 + wave) * (16 * TILES);
  const bool full = wave_key0 + 16 * TILES <= a.n;  // uniform: no key of this wavefront is past the end
  const int64_t wrow0 = gbase + wave_key0;
  u32x4 ci[ROUNDS][NI > 0 ? NI : 1], cq[ROUNDS][NQ > 0 ? NQ : 1];
  float cg[ROUNDS][NR], cn[ROUNDS][NR];
  const u32x4* const idx16 = reinterpret_cast<const u32x4*>(a.idx);
  const u32x4* const qjl16 = reinterpret_cast<const u32x4*>(a.qjl);
  const int64_t idx_last = a.total_rows * BITS - 1, qjl_last = a.total_rows - 1;  // last 16-byte piece
  auto in_round = [&](int i, int count) {  // piece i * 64 + lane of a round's `count` pieces, the last one repeated
    const int p = i * 64 + lane;
    return count % 64 == 0 ? p : (p < count ? p : count - 1);
  };
  auto issue_round = [&](int r) {
    const int64_t row0 = wrow0 + r * ROWS;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      int64_t piece = row0 * BITS + in_round(i, PI);
      if (!full) piece = piece < idx_last ? piece : idx_last;
      ci[r][i] = idx16[piece];
    }
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
      int64_t piece = row0 + in_round(i, ROWS);
      if (!full) piece = piece < qjl_last ? piece : qjl_last;
      cq[r][i] = qjl16[piece];
    }
#pragma unroll
    for (int i = 0; i < NR; ++i) {
      int64_t row = row0 + in_round(i, ROWS);
      if (!full) row = row < a.total_rows - 1 ? row : a.total_rows - 1;
      cg[r][i] = PROD ? a.gamma[row] : 0.f;
      cn[r][i] = a.norm != nullptr ? a.norm[row] : 1.f;
    }
  };
  constexpr int AHEAD = (INFLIGHT > 0 && INFLIGHT < ROUNDS) ? INFLIGHT : ROUNDS;  // rounds requested before the first is used
#pragma unroll
  for (int r = 0; r < AHEAD; ++r) issue_round(r);

  // ---- 3. rotate / sketch this workgroup's four queries, 4. fixed point --------------------------
  prep.matvec(a, group, q0, part_s);
  __syncthreads();
  i8_digitise_terms<BITS, PROD>(a, q0, wave, lane, part_s, dig_s, scal_s);
  __syncthreads();  // digits and scalars are in LDS

  // ---- 5. A operands: lane = row + 16 kq, row = 4 * query + digit; one image per masked sum --------
  const int a_query = col >> 2, a_digit = col & 3;
  constexpr bool A_REGS = NTA <= 3;  // else read at every use (LDS has nothing else to do)
  auto a_read = [&](int j, int s) -> v4i {
    return *reinterpret_cast<const v4i*>(dig_s + ((j * 4 + a_query) * 4 + a_digit) * 128 + (s * 4 + kq) * 16);  // slot order of i8_shifted_slot
  };
  v4i areg[A_REGS ? NTA : 1][2];
  if (A_REGS) {
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int s = 0; s < 2; ++s) areg[j][s] = a_read(j, s);
  }
  float r_inv = 0.f, base_r = 0.f, s_inv = 0.f, s_sum = 0.f;
  if (BITS > 0) {
    r_inv = scal_s[(0 * 4 + kq) * 4];
    base_r = scal_s[(0 * 4 + kq) * 4 + 1];
  }
  if (PROD) {
    s_inv = scal_s[(1 * 4 + kq) * 4];
    s_sum = scal_s[(1 * 4 + kq) * 4 + 1];
  }

  // B operand of k-step s from the 32 stored bits w of this lane's k-chunk: dword i keeps bits
  // 4 s + i + {0, 8, 16, 24} of w where they are, one AND each.  Byte b of it is bit
  // k + 8 b (k = 4 s + i) times 2^k; the digits on the A side are those of the coordinate
  // times 2^(7 - k) (negated for k = 7, where the byte reads as -128), so every product
  // carries the same factor 128.
  auto expand16 = [&](uint32_t w, int s) -> v4i {
    v4i b;
#pragma unroll
    for (int i = 0; i < 4; ++i) b[i] = (int)(w & (0x01010101u << (4 * s + i)));
    return b;
  };
  auto digits_sum = [&](const v4i& acc) -> float {  // (D0 + 2^7 D1 + 2^14 D2 + 2^21 D3) / 128, D0 a multiple of 128
    return (float)((((acc[3] << 7) + acc[2]) << 7) + acc[1] + (acc[0] >> 7));
  };

  const float zs = 2.f * s_inv;

  // ---- 6. tiles ------------------------------------------------------------------------------
  // A four-stage software pipeline written out in source order: the words of tile t+2 are
  // fetched from the staging region, the mask operands of tile t+1 are made, the MFMAs of
  // tile t run and the sums of tile t-1 are combined and stored.  The staging region is
  // private to the wavefront and LDS executes a wavefront's instructions in order, so the
  // next round may be written as soon as the last word fetch of the current one is issued.
  // words of four tiles in flight (ring indexed by tile % 4)
  uint32_t wp[4][NW], wz[4];
  float wkg[4], wnu[4];
  auto put_round = [&](int r) {
#pragma unroll
    for (int i = 0; i < NI; ++i) *reinterpret_cast<u32x4*>(stage + IDX_OFF + in_round(i, PI) * 16) = ci[r][i];
#pragma unroll
    for (int i = 0; i < NQ; ++i) *reinterpret_cast<u32x4*>(stage + QJL_OFF + in_round(i, ROWS) * 16) = cq[r][i];
#pragma unroll
    for (int i = 0; i < NR; ++i) {
      if (PROD) *reinterpret_cast<float*>(stage + GAM_OFF + in_round(i, ROWS) * 4) = cg[r][i];
      *reinterpret_cast<float*>(stage + NRM_OFF + in_round(i, ROWS) * 4) = cn[r][i];
    }
  };
  auto fetch = [&](int t) {
    const int lr = (t % RT) * 16 + col;  // row within the staged round
#pragma unroll
    for (int pl = 0; pl < BITS; ++pl)
      wp[t & 3][pl] = *reinterpret_cast<const uint32_t*>(stage + IDX_OFF + ((lr * 4 + kq) * BITS + pl) * 4);
    wz[t & 3] = PROD ? *reinterpret_cast<const uint32_t*>(stage + QJL_OFF + (lr * 4 + kq) * 4) : 0u;
    wkg[t & 3] = PROD ? *reinterpret_cast<const float*>(stage + GAM_OFF + lr * 4) : 0.f;
    wnu[t & 3] = *reinterpret_cast<const float*>(stage + NRM_OFF + lr * 4);
  };
  auto lookups = [&](int t, int s, v4i (&b)[NTA]) {  // B operands of k-step s of tile t
    int j = 0;
#pragma unroll
    for (int m = 1; m <= NM; ++m) {
      if (!i8_term(m)) continue;
      uint32_t x = 0u;
#pragma unroll
      for (int pl = 0; pl < BITS; ++pl)
        if (m & (1 << pl)) x ^= wp[t & 3][pl];
      b[j++] = expand16(x, s);
    }
    if (PROD) b[j] = expand16(wz[t & 3], s);
  };
  // all masked sums of the rotated query go to accumulator 0, the sketch's to the last one
  constexpr int NACC = (BITS > 0 ? 1 : 0) + (PROD ? 1 : 0);
  auto mfmas = [&](int s, const v4i (&b)[NTA], v4i (&c)[NACC]) {
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int to = (PROD && j == NT - 1) ? NACC - 1 : 0;
      c[to] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A_REGS ? areg[A_REGS ? j : 0][s] : a_read(j, s), b[j], c[to], 0, 0, 0);
    }
  };
  // with few masked sums per tile the operands of the next tile are looked up while this
  // tile's MFMAs run; with many there are no registers for that
  constexpr bool PIPE = NTA <= 3;
  auto run_tiles = [&](auto full_c) {
    constexpr bool FULL = decltype(full_c)::value;
    v4i bop[PIPE ? 2 : 1][2][NTA];
    v4i acc[2][NACC];
    auto finish = [&](int t) {
      const v4i(&c)[NACC] = acc[t & 1];
      float total = BITS > 0 ? fmaf(r_inv, digits_sum(c[0]), base_r) : 0.f;
      if (PROD) total = fmaf(a.kappa * wkg[t & 3], fmaf(zs, digits_sum(c[NACC - 1]), -s_sum), total);
      total *= wnu[t & 3];
      sink(t, total, FULL || wave_key0 + t * 16 + col < a.n);
    };
    // everything needed before tile t's words can be fetched
    auto stage_for = [&](int t) {
      if (t % RT == 0) {
        put_round(t / RT);
        if (t / RT + AHEAD < ROUNDS) issue_round(t / RT + AHEAD);
      }
    };
    stage_for(0);
    fetch(0);
    if (PIPE) {
      lookups(0, 0, bop[0][0]);
      lookups(0, 1, bop[0][1]);
    }
    stage_for(1);
    fetch(1);
    // tiles that have at least one key (uniform over the wavefront)
    const int live_tiles = FULL ? TILES : (int)((a.n - wave_key0 + 15) >> 4);
#pragma unroll
    for (int t = 0; t < TILES; ++t) {
      if (FULL || t < live_tiles) {
        if (t + 2 < TILES) {
          stage_for(t + 2);
          fetch(t + 2);
        }
#pragma unroll
        for (int j = 0; j < NACC; ++j) acc[t & 1][j] = v4i{0, 0, 0, 0};
        if (PIPE) {
          if (t + 1 < TILES) {
            lookups(t + 1, 0, bop[(t + 1) & 1][0]);
            lookups(t + 1, 1, bop[(t + 1) & 1][1]);
          }
          mfmas(0, bop[t & 1][0], acc[t & 1]);
          mfmas(1, bop[t & 1][1], acc[t & 1]);
        } else {
          lookups(t, 0, bop[0][0]);
          lookups(t, 1, bop[0][1]);
          mfmas(0, bop[0][0], acc[t & 1]);
          mfmas(1, bop[0][1], acc[t & 1]);
        }
      }
      if (t > 0 && (FULL || t - 1 < live_tiles)) finish(t - 1);
    }
    if (FULL || TILES - 1 < live_tiles) finish(TILES - 1);
  };
  if (full) run_tiles(std::true_type{});
  else run_tiles(std::false_type{});
}

}  // namespace tq
