// Many queries per code (nearest-neighbour search, Sec. 4.4): the estimator of Sec. 3.2 for a block of
// queries against a block of codes is a dense contraction whose code-side operand takes few values,
//     score[m][i] = nu_i * ( sum_j qr[m][j] c[idx_ij]  +  kappa gamma_i sum_j qs[m][j] z_ij ).
// It runs on the bf16 matrix cores (16 x the fp32 rate): every fp32 factor is taken as its two leading bf16
// pieces, x ~ x1 + x2 (8 + 8 significant bits and a sign: what is left is below 2^-17 |x|), a product of two pieces is
// exact in fp32, and the MFMA accumulates in fp32.  The three piece products of combined weight >= 2^-9 are
// kept,
//     q c ~ q1 c1 + q1 c2 + q2 c1,
// so a term is off by 2^-17.8 |q| |c| in the root mean square (2^-15 if both factors sit at the bottom of their
// binades and every dropped part has its largest size).  Over the d terms of a score these errors average out: the
// scores are within about 2e-7 |q| nu of the exact ones; a single dequantised coordinate (the transposed mode,
// one term per coordinate and query) within about 2e-5 of its typical size.  Sign operands need one piece:
// z = +-1 is a bf16 value, and a 1-bit codebook is +-c_1 with c_1 applied after the sum; those products take
// two MFMAs (q1, q2).
//
// Workgroup = 512 threads = 8 wavefronts, tile 128 or 256 queries x 256 or 128 codes, k in steps of 16 (one
// v_mfma_f32_32x32x16_bf16 per piece product and 32 x 32 sub-tile), operands through two LDS buffers with a
// 48-byte row stride (conflict-free 16-byte reads).  Queries are split into pieces while they are staged
// (read as fp32: 4 bytes per element instead of 6); codes are decoded into pieces while they are staged
// (bit planes -> bucket number -> table of pieces in LDS, or straight to +-1).  Wavefront (wm, wn) owns rows
// 64 wm .. and columns 64 wn .. of the tile: 2 x 2 sub-tiles, one accumulator set per segment (the sign
// segment is scaled per code by kappa gamma, so it cannot share the accumulator of the first).
//
// Top-k without a score matrix (TOPK): a workgroup owns one block of queries and a contiguous range of code
// tiles, which it walks with the k-loop above.  Every query row has RS (score, index) slots in LDS: the k best
// pairs so far, sorted, and behind them an append area with a counter.  After a tile, a score that reaches its
// row's k-th best is appended (one LDS atomic for the position; all wavefronts at once); in the steady state
// that is one compare per score and a handful of appends per tile.  Then the half-waves share out the rows:
// a row with appended pairs has each of its <= 32 pairs ranked against the others by one lane each, and the
// pairs of rank < k written to their slots, which also gives the row's new bar.  Scores that found the append
// area full stay in their registers and the round is repeated with the raised bars (only the first tiles of a
// range need that).  The lists of all ranges are then joined by topk_merge_kernel.  Order everywhere: larger
// score first, equal scores by lower index, so the result is the one a full sort of the score matrix gives.
#include <cstring>

#include "tq_bf3.h"

namespace tq {

namespace {

constexpr int KL = 16;       // largest k of the fused top-k

__device__ __forceinline__ bool better(float va, int ia, float vb, int ib) {
  return va > vb || (va == vb && ia < ib);
}


constexpr int KT = 16;  // k per step; queries per tile TM: 128 or 256, codes per tile TN: 256 or 128 (template parameters)
constexpr int LDK = 24;      // bf16 per LDS row: 16 used + 8 padding = 48 bytes
constexpr int SPAN = 4;      // coordinate groups (of 32) whose plane words a thread holds at a time
constexpr int QP = 2;        // leading bf16 pieces kept of a query coordinate (and of a centroid)

template <int BITS, bool PROD, int TM, int TN>
struct Cfg {
  static constexpr int WM = TM / 64, WN = 8 / WM;  // wavefronts along the queries / the codes
  static constexpr int CT = TN / (32 * WN);        // 32-column sub-tiles of a wavefront (2 row sub-tiles always)
  static constexpr int PC = BITS == 0 ? 0 : BITS == 1 ? 1 : QP;  // pieces of a decoded centroid
  static constexpr int SEGS = (BITS > 0 ? 1 : 0) + (PROD ? 1 : 0);
  static constexpr int A_ELEMS = SEGS * QP * TM * LDK;
  static constexpr int B_ELEMS = (PC + (PROD ? 1 : 0)) * TN * LDK;
  static constexpr int BUF_ELEMS = A_ELEMS + B_ELEMS;
  static constexpr int LDS_BYTES = 2 * BUF_ELEMS * 2 + 16 * 8;  // two buffers, then the piece table
  // fused top-k: per query row RS (score, index) slots (the sorted k best, then the append area), a counter per
  // row, and the two "some score is still waiting" flags
  static constexpr int RS = TM == 256 ? 26 : 32;  // at most 32: one lane of a half-wave per pair when a row is ranked
  static constexpr int LDS_BYTES_TOPK = LDS_BYTES + TM * RS * 8 + TM * 4 + 16;
  static constexpr bool FITS = LDS_BYTES_TOPK <= 156 * 1024;
};

struct Bf3Args {
  const float* qr;  // [groups * M][d] rotated queries
  const float* qs;  // [groups * M][d] sketched queries (PROD)
  int M;            // queries per group
  int d;
  const uint32_t* idx;
  const uint32_t* qjl;
  const float* gamma;
  const float* norm;  // nullable: unit-norm codes
  int64_t n;          // codes per group
  float* out;         // [groups * M][ldo]; transposed: [groups * n][ldo], M values per code
  int64_t ldo;
  int transposed;
  float kappa;
  Codebook cb;
  // fused top-k (TOPK kernels): workgroup w of a 1-D grid owns query block w_qb and code tiles [t0, t1) of range w_r
  int topk;          // 1..KL
  int groups;
  int ranges;        // code-tile ranges per query block
  int qblocks;       // query blocks per group
  int tiles_n;       // code tiles per group
  int xcd_split;     // fused top-k: ranges per XCD (0: no split by XCD); plain kernel: 1 = query block fastest
  float* part_val;   // [groups * M][ranges][topk]
  int32_t* part_idx;
};

template <int BITS, bool PROD, int TM, int TN, bool TOPK>
__global__ __launch_bounds__(512) void score_bf3_kernel(const Bf3Args a) {
  using C = Cfg<BITS, PROD, TM, TN>;
  constexpr int CP = TN / 32;  // coordinates of one code a thread decodes per step: 8 or 4
  constexpr int PC = C::PC;
  constexpr int CT = C::CT;
  constexpr int AR = TM / 128;  // 16-byte pieces of a query tile row set a thread stages per segment
  constexpr int NB = BITS > 0 ? BITS : 1;
  constexpr bool PIN = !(TOPK && PROD);  // see the k-loop
  extern __shared__ __attribute__((aligned(16))) unsigned short lds_s[];
  constexpr int STAGE_ELEMS = 2 * C::BUF_ELEMS;
  uint2* const table_s = reinterpret_cast<uint2*>(lds_s + STAGE_ELEMS);  // [16]: pieces of centroid k

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % C::WM, wn = wave / C::WM;
  const int gw = a.d >> 5;  // coordinate groups per code
  int group, m0, range = 0;
  int64_t tile_begin, tile_end;
  if (TOPK) {
    // workgroup -> (query block, range).  Workgroups are dealt to the 8 XCDs in turn; with xcd_split (=
    // ranges / 8) the query blocks that walk the same range of codes sit on one XCD and share its L2
    const int w = blockIdx.x;
    const int nqb = a.qblocks * a.groups;
    int qb;
    if (a.xcd_split > 0) {
      // XCD w % 8 takes ranges / 8 consecutive ranges, each with all of its query blocks
      const int slot = w / 8;
      qb = slot % nqb;
      range = (w % 8) * a.xcd_split + slot / nqb;
    } else {
      qb = w % nqb;
      range = w / nqb;
    }
    // (the results of integer divisions are pinned to scalar registers: the compiler takes them for per-lane
    // values otherwise, and with them every address of the k-loop and the epilogue)
    range = __builtin_amdgcn_readfirstlane(range);
    group = __builtin_amdgcn_readfirstlane(qb / a.qblocks);
    m0 = __builtin_amdgcn_readfirstlane((qb % a.qblocks) * TM);
    tile_begin = __builtin_amdgcn_readfirstlane((int)((int64_t)range * a.tiles_n / a.ranges));
    tile_end = __builtin_amdgcn_readfirstlane((int)((int64_t)(range + 1) * a.tiles_n / a.ranges));
  } else {
    // workgroup -> tile.  Workgroups are dealt to the 8 XCDs in turn; every XCD gets a contiguous range of
    // tiles.  With xcd_split the query block runs fastest, so the query blocks that read the same block of
    // codes share one L2 and run at about the same time: dequantisation (d / TM "query" blocks per block of
    // codes, C5: 88 -> 72 ms) and scoring with more than four query blocks (C5 shape: 29 -> 24 ms); with
    // four 256-row blocks the order below is the faster one (C4 shape: 9.6 against 10.7 ms)
    group = blockIdx.z;
    if (a.xcd_split > 0) {
      // (32-bit unsigned arithmetic, and the results pinned to scalar registers: a division makes the compiler
      // treat them as per-lane values, and with them every address of the k-loop and the epilogue)
      const uint32_t qblocks = (uint32_t)(a.M + TM - 1) / TM;
      const uint32_t total = qblocks * (uint32_t)a.tiles_n;  // below 2^31: checked at launch
      const uint32_t per_xcd = (total + 7u) / 8u;
      const uint32_t logical = (blockIdx.x % 8u) * per_xcd + blockIdx.x / 8u;
      if (logical >= total) return;  // the whole workgroup
      m0 = __builtin_amdgcn_readfirstlane((int)(logical % qblocks) * TM);
      tile_begin = __builtin_amdgcn_readfirstlane((int)(logical / qblocks));
    } else {
      // a grid of (blocks of codes, query blocks): the workgroups in flight write neighbouring pieces of the
      // same score rows
      m0 = blockIdx.y * TM;
      tile_begin = blockIdx.x;
    }
    tile_end = tile_begin + 1;
  }
  // fused top-k state, behind the staging buffers and the piece table
  // [TM][RS] (score bits, index): slots [0, k) sorted, best first; slots [k, RS) appended since the last ranking
  constexpr int RS = C::RS;
  uint2* const list = reinterpret_cast<uint2*>(lds_s + STAGE_ELEMS + 64);
  int* const cnt_s = reinterpret_cast<int*>(list + TM * RS);  // [TM] pairs appended (may count past the area's end)
  int* const wait_s = cnt_s + TM;                             // [2] a score found its row's area full (by round parity)
  const float NEG = -__builtin_inff();
  const uint2 NONE = make_uint2(__float_as_uint(NEG), 0x7fffffffu);  // "no pair": worse than any score
  if (TOPK) {
    for (int e = tid; e < TM * RS; e += 512) list[e] = NONE;
    for (int e = tid; e < TM + 2; e += 512) cnt_s[e] = 0;
  }

  if (PC == QP && tid < 16) {
    uint32_t p1, p2, p3;
    split3(a.cb.c[tid], p1, p2, p3);
    table_s[tid] = make_uint2(p1 | (p2 << 16), p3);
  }

  for (int64_t tile = tile_begin; tile < tile_end; ++tile) {
  // In the tile loop of the fused top-k everything derived from the thread's number is made again per tile:
  // computed once ahead of the loop, the dozens of LDS and global addresses of the k-loop would stay in
  // registers through the epilogue and the selection, which need them for the scores.
  int ttid = tid;
  if (TOPK) asm volatile("" : "+v"(ttid));
  const int tlane = ttid & 63;

  // ---- staging roles --------------------------------------------------------------------------------
  // A: thread = (row tid / 4, four consecutive k at 4 (tid % 4)) of each segment
  // (and of row + 128 when the tile has 256 rows)
  const int a_row = ttid >> 2, a_k = (ttid & 3) * 4;
  const float* a_src0[AR];
  const float* a_src1[AR];
#pragma unroll
  for (int i = 0; i < AR; ++i) {
    const int r = m0 + a_row + 128 * i < a.M ? m0 + a_row + 128 * i : a.M - 1;  // clamped: such rows are not stored
    a_src0[i] = a.qr + ((int64_t)group * a.M + r) * a.d + a_k;
    a_src1[i] = PROD ? a.qs + ((int64_t)group * a.M + r) * a.d + a_k : nullptr;
  }
  // B: thread = (code tid % TN, CP consecutive k at CP (tid / TN)); the code changes with the tile
  const int b_col = ttid % TN, b_part = ttid / TN;
  const uint32_t* b_idx = nullptr;
  const uint32_t* b_qjl = nullptr;

  f32x4 areg[2][AR];
  uint32_t wcur[SPAN][NB], zcur[SPAN], wnxt[SPAN][NB], znxt[SPAN];
  auto load_a = [&](int step) {
#pragma unroll
    for (int i = 0; i < AR; ++i) {
      if (BITS > 0) areg[0][i] = *reinterpret_cast<const f32x4*>(a_src0[i] + step * KT);
      if (PROD) areg[1][i] = *reinterpret_cast<const f32x4*>(a_src1[i] + step * KT);
    }
  };
  auto load_words = [&](int span) {  // plane words of coordinate groups [SPAN span, SPAN span + SPAN)
#pragma unroll
    for (int g = 0; g < SPAN; ++g) {
      const int gg = SPAN * span + g < gw ? SPAN * span + g : gw - 1;  // clamped: never decoded
#pragma unroll
      for (int pl = 0; pl < BITS; ++pl) wnxt[g][pl] = b_idx[gg * BITS + pl];
      znxt[g] = PROD ? b_qjl[gg] : 0u;
    }
  };
  auto store_a = [&](unsigned short* buf) {
    int seg = 0;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      if (s == 0 ? BITS == 0 : !PROD) continue;
#pragma unroll
      for (int i = 0; i < AR; ++i) {
        uint32_t lo[3], hi[3];
        split3_pair(f32x2{areg[s][i][0], areg[s][i][1]}, lo[0], lo[1], lo[2]);
        split3_pair(f32x2{areg[s][i][2], areg[s][i][3]}, hi[0], hi[1], hi[2]);
#pragma unroll
        for (int pc = 0; pc < QP; ++pc)
          *reinterpret_cast<uint2*>(buf + ((seg * QP + pc) * TM + a_row + 128 * i) * LDK + a_k) = make_uint2(lo[pc], hi[pc]);
      }
      ++seg;
    }
  };
  // CP sign bits -> CP bf16 values +-1 (bit set: +1), two per word
  auto signs = [&](uint32_t bits, uint32_t (&v)[CP / 2]) {
#pragma unroll
    for (int e = 0; e < CP / 2; ++e)
      v[e] = 0xBF80BF80u ^ (((bits >> (2 * e)) & 1u) << 15) ^ (((bits >> (2 * e + 1)) & 1u) << 31);
  };
  auto put = [&](unsigned short* dst, const uint32_t (&v)[CP / 2]) {  // CP bf16 values: 16 or 8 bytes
    if (CP == 8) *reinterpret_cast<u32x4*>(dst) = u32x4{v[0], v[1], v[CP / 2 - 2], v[CP / 2 - 1]};
    else *reinterpret_cast<uint2*>(dst) = make_uint2(v[0], v[1]);
  };
  auto store_b = [&](unsigned short* buf, int j) {  // j: step within its span of 2 SPAN steps (a constant at every call)
    unsigned short* const bb = buf + C::A_ELEMS;
    const int g = j >> 1, off = (j & 1) * 16 + CP * b_part;  // word of the span, first bit
    if (PC == 1) {
      uint32_t v[CP / 2];
      signs(wcur[g][0] >> off, v);
      put(bb + b_col * LDK + CP * b_part, v);
    } else if (PC == QP) {
      uint32_t lv[CP / 4];  // bucket numbers of 4 coordinates, one per byte
#pragma unroll
      for (int h = 0; h < CP / 4; ++h) {
        lv[h] = 0u;
#pragma unroll
        for (int pl = 0; pl < BITS; ++pl)
          lv[h] |= ((((wcur[g][pl] >> (off + 4 * h)) & 0xFu) * 0x00204081u) & 0x01010101u) << pl;
      }
      uint2 e[CP];
#pragma unroll
      for (int u = 0; u < CP; ++u) e[u] = table_s[(lv[u >> 2] >> (8 * (u & 3))) & 0xFFu];
      uint32_t v1[CP / 2], v2[CP / 2];
#pragma unroll
      for (int u = 0; u < CP / 2; ++u) {
        v1[u] = __builtin_amdgcn_perm(e[2 * u + 1].x, e[2 * u].x, 0x05040100u);  // low halves: first pieces
        v2[u] = __builtin_amdgcn_perm(e[2 * u + 1].x, e[2 * u].x, 0x07060302u);  // high halves: second pieces
      }
      put(bb + (0 * TN + b_col) * LDK + CP * b_part, v1);
      put(bb + (1 * TN + b_col) * LDK + CP * b_part, v2);
    }
    if (PROD) {
      uint32_t v[CP / 2];
      signs(zcur[g] >> off, v);
      put(bb + (PC * TN + b_col) * LDK + CP * b_part, v);
    }
  };
  auto take_words = [&]() {
#pragma unroll
    for (int g = 0; g < SPAN; ++g) {
#pragma unroll
      for (int pl = 0; pl < BITS; ++pl) wcur[g][pl] = wnxt[g][pl];
      zcur[g] = znxt[g];
    }
  };

  const int f_row = tlane & 31, f_k = (tlane >> 5) * 8;  // fragment: row / column within a sub-tile, first k
  unsigned short* const buf0 = lds_s;
  unsigned short* const buf1 = lds_s + C::BUF_ELEMS;
  const int steps = a.d / KT;
  const int spans = steps / (2 * SPAN);

  const int64_t n0 = tile * TN;
  {
    const int64_t b_row = (int64_t)group * a.n + (n0 + b_col < a.n ? n0 + b_col : a.n - 1);
    b_idx = a.idx + b_row * ((int64_t)gw * BITS);
    b_qjl = PROD ? a.qjl + b_row * gw : nullptr;
  }
  floatx16 acc1[2][CT], acc2[2][PROD ? CT : 1];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt)
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        acc1[rt][ct][r] = 0.f;
        if (PROD) acc2[rt][ct][r] = 0.f;
      }

  auto compute = [&](const unsigned short* buf) {
    const unsigned short* const bb = buf + C::A_ELEMS;
    auto frag = [&](const unsigned short* base, int row) -> bf16x8 {
      return *reinterpret_cast<const bf16x8*>(base + row * LDK + f_k);
    };
    int seg = 0;
    if (BITS > 0) {
      bf16x8 af[2][QP], bf[CT][PC > 0 ? PC : 1];
#pragma unroll
      for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int pc = 0; pc < QP; ++pc) af[rt][pc] = frag(buf + (seg * QP + pc) * TM * LDK, 64 * wm + 32 * rt + f_row);
#pragma unroll
      for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int pc = 0; pc < PC; ++pc) bf[ct][pc] = frag(bb + pc * TN * LDK, 32 * CT * wn + 32 * ct + f_row);
      // piece products outermost: consecutive MFMAs go to different accumulators; smallest products first
      constexpr int NTERM = PC == 1 ? QP : 3;
      constexpr int TA[3] = {1, 0, 0};                          // query piece of each product
      constexpr int TB[3] = {0, 1, 0};                          // centroid piece
#pragma unroll
      for (int t = 0; t < NTERM; ++t)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
          for (int ct = 0; ct < CT; ++ct)
            acc1[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[rt][PC == 1 ? QP - 1 - t : TA[t]], bf[ct][PC == 1 ? 0 : TB[t]],
                                                                   acc1[rt][ct], 0, 0, 0);
      ++seg;
    }
    if (PROD) {
      bf16x8 af[2][QP], bf[CT];
#pragma unroll
      for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int pc = 0; pc < QP; ++pc) af[rt][pc] = frag(buf + (seg * QP + pc) * TM * LDK, 64 * wm + 32 * rt + f_row);
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) bf[ct] = frag(bb + PC * TN * LDK, 32 * CT * wn + 32 * ct + f_row);
#pragma unroll
      for (int pc = QP - 1; pc >= 0; --pc)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
          for (int ct = 0; ct < CT; ++ct)
            acc2[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[rt][pc], bf[ct], acc2[rt][ct], 0, 0, 0);
    }
  };

  // ---- k loop: one barrier per step ----------------------------------------------------------------
  load_a(0);
  load_words(0);
  take_words();
  __syncthreads();  // the piece table (and, from the second tile on, the end of the previous tile's selection)
  store_a(buf0);
  store_b(buf0, 0);
  __syncthreads();
  // whole spans: no branch inside a step; after the last step the same step is staged once more, unused
  for (int sp = 0; sp < spans; ++sp) {
#pragma unroll
    for (int j = 0; j < 2 * SPAN; ++j) {  // unrolled, so that the plane words are picked by constant indices
      const int s = sp * (2 * SPAN) + j;
      load_a(s + 1 < steps ? s + 1 : s);
      if (j == 0) load_words(sp + 1);  // requested a span ahead (clamped past the end)
      // The staging arithmetic is kept out of the MFMAs of a step (the scheduler interleaves them in most
      // instantiations, and the same instructions then take 3-12 % longer: C5 dequantise 88 -> 79 ms).  The
      // two-segment kernels of the fused top-k are left alone: their register pressure keeps the scheduler
      // from interleaving anyway, and pinned they lose the overlap of a step's last MFMAs with the next
      // step's reads (C5 score + top-10: 25.2 against 26.2 ms).
      if (PIN) __builtin_amdgcn_sched_barrier(0);
      compute((j & 1) ? buf1 : buf0);
      if (PIN) __builtin_amdgcn_sched_barrier(0);
      if (j == 2 * SPAN - 1) take_words();
      store_a((j & 1) ? buf0 : buf1);
      store_b((j & 1) ? buf0 : buf1, (j + 1) & (2 * SPAN - 1));
      __syncthreads();
    }
  }
  // the steps of an incomplete last span (d not a multiple of 128)
  for (int sp = spans; sp * (2 * SPAN) < steps; ++sp) {
#pragma unroll
    for (int j = 0; j < 2 * SPAN; ++j) {
      const int s = sp * (2 * SPAN) + j;
      if (s < steps) {  // uniform
        const bool more = s + 1 < steps;
        if (more) load_a(s + 1);
        if (j == 0 && more) load_words(sp + 1);
        if (PIN) __builtin_amdgcn_sched_barrier(0);
        compute((j & 1) ? buf1 : buf0);
        if (PIN) __builtin_amdgcn_sched_barrier(0);
        if (more) {
          if (j == 2 * SPAN - 1) take_words();
          store_a((j & 1) ? buf0 : buf1);
          store_b((j & 1) ? buf0 : buf1, (j + 1) & (2 * SPAN - 1));
        }
        __syncthreads();
      }
    }
  }

  // ---- epilogue: per-code factors, store -----------------------------------------------------------
  const float c1 = BITS == 1 ? a.cb.c[1] : 1.f;
  // Where the selection keeps the finished scores.  With 128-row tiles there is room for registers of their
  // own (the accumulators' life then ends with this epilogue); the 256-row tile has none to spare and keeps
  // them in the accumulator registers, which the selection then only reads (marking appended scores there
  // would carry the accumulators through the selection's rounds and cost copies in the k-loop).  Measured,
  // each tile shape is 10-15 % slower with the other choice.
  constexpr bool SEL_COPY = TOPK && TM == 128;
  float sv[SEL_COPY ? 2 : 1][SEL_COPY ? CT : 1][SEL_COPY ? 16 : 1];
  // in the tile loop of the fused top-k the epilogue's addresses must not be computed ahead of the loop (they
  // would be carried through it in registers the k-loop needs): lane-derived values are re-made per tile
  int e_row = f_row, e_half = lane >> 5;
  if (TOPK) asm volatile("" : "+v"(e_row), "+v"(e_half));
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    const int64_t col = n0 + 32 * CT * wn + 32 * ct + e_row;
    const bool col_live = col < a.n;
    const int64_t crow = (int64_t)group * a.n + (col_live ? col : a.n - 1);
    const float nu = a.norm != nullptr ? a.norm[crow] : 1.f;
    const float kg = PROD ? a.kappa * a.gamma[crow] : 0.f;
    if (a.transposed) {
      // one row per code (dequantisation: the "queries" are the rows of Pi^T, the result is x~): a lane owns
      // four consecutive values of its code's row per accumulator quad
      float* const orow = a.out + crow * a.ldo;
#pragma unroll
      for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
          const int row = m0 + 64 * wm + 32 * rt + 8 * qd + 4 * e_half;
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e)
            v[e] = nu * fmaf(kg, PROD ? acc2[rt][ct][4 * qd + e] : 0.f, c1 * acc1[rt][ct][4 * qd + e]);
          if (col_live && row + 3 < a.M) {
            *reinterpret_cast<f32x4*>(orow + row) = v;
          } else if (col_live) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (row + e < a.M) orow[row + e] = v[e];
          }
        }
      continue;
    }
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + 64 * wm + 32 * rt + 8 * (r >> 2) + (r & 3) + 4 * e_half;
        const float v = nu * fmaf(kg, PROD ? acc2[rt][ct][r] : 0.f, c1 * acc1[rt][ct][r]);
        const bool live = col_live && row < a.M;
        if (live && (!TOPK || a.out != nullptr)) a.out[((int64_t)group * a.M + row) * a.ldo + col] = v;
        // what is not a score becomes NaN, which no comparison lets in
        if (SEL_COPY) sv[SEL_COPY ? rt : 0][SEL_COPY ? ct : 0][SEL_COPY ? r : 0] = live ? v : __builtin_nanf("");
        else if (TOPK) acc1[rt][ct][r] = live ? v : __builtin_nanf("");
      }
  }

  // ---- selection: the tile's scores against the k best of every query row so far ----------------------
  if (TOPK) {
    const int half = e_half;
    const int kk = a.topk;
    const int area = RS - kk;  // append slots per row
    const bool last_tile = tile + 1 == tile_end;
    int round = 0;
    bool again;
    // scores that have been appended: NaN in their own registers, or (scores in the accumulators) bit
    // 16 (ct % 2) + r of word [rt][ct / 2]
    uint32_t done[2][(CT + 1) / 2];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
      for (int w = 0; w < (CT + 1) / 2; ++w) done[rt][w] = 0u;
    do {
      // every row's k-th best score, fetched in one batch (a fetch per compare would leave each compare
      // waiting for LDS)
      bool waiting = false;
#pragma unroll
      for (int rt = 0; rt < 2; ++rt) {
        float bar[16];
#pragma unroll
        for (int r = 0; r < 16; ++r)
          bar[r] = __uint_as_float(list[(64 * wm + 32 * rt + 8 * (r >> 2) + (r & 3) + 4 * half) * RS + kk - 1].x);
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
          const int col = (int)n0 + 32 * CT * wn + 32 * ct + e_row;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float v = SEL_COPY ? sv[SEL_COPY ? rt : 0][SEL_COPY ? ct : 0][SEL_COPY ? r : 0] : acc1[rt][ct][r];
            const uint32_t bit = 1u << (16 * (ct & 1) + r);
            if (v >= bar[r] && (SEL_COPY || (done[rt][ct >> 1] & bit) == 0u)) {  // NaN never passes
              const int lrow = 64 * wm + 32 * rt + 8 * (r >> 2) + (r & 3) + 4 * half;
              const int pos = atomicAdd(&cnt_s[lrow], 1);
              if (pos < area) {
                list[lrow * RS + kk + pos] = make_uint2(__float_as_uint(v), (uint32_t)col);
                if (SEL_COPY) sv[SEL_COPY ? rt : 0][SEL_COPY ? ct : 0][SEL_COPY ? r : 0] = __builtin_nanf("");
                else done[rt][ct >> 1] |= bit;
              } else {
                waiting = true;  // kept for the next round, when the row's bar is higher
              }
            }
          }
        }
      }
      if (waiting) wait_s[round & 1] = 1;
      __syncthreads();
      // ranking: half-wave hw takes rows hw, hw + 16, ...; lane l of the half-wave is pair l of the row.  A row
      // is ranked once its area is half full (its bar is stale until then, which only lets a few more scores
      // in), and at the end of the range.
      {
        const int hw = 2 * wave + half, l = lane & 31;
        int mine_c = l < TM / 16 ? cnt_s[hw + 16 * l] : 0;  // lane l: pairs waiting in row hw + 16 l
        mine_c = mine_c < area ? mine_c : area;
        const bool due = mine_c > 0 && (2 * mine_c >= area || last_tile);
        const unsigned long long due64 = __ballot(due);
        uint32_t rows_due = ((uint32_t)due64 | (uint32_t)(due64 >> 32)) & 0xffffu;  // rows due in either half-wave
        const uint32_t due_half = half ? (uint32_t)(due64 >> 32) : (uint32_t)due64;
        while (rows_due != 0u) {  // uniform
          const int i = __builtin_ctz(rows_due);
          rows_due &= rows_due - 1u;
          const int c_i = __shfl(mine_c, (lane & 32) + i);  // by every lane: the exchange is not to run under a mask
          const int c = ((due_half >> i) & 1u) ? c_i : 0;
          uint2* const row = list + (hw + 16 * i) * RS;
          const int n_ent = c > 0 ? kk + c : 0;
          const uint2 mine = l < n_ent ? row[l] : NONE;
          int rank = 0;
#pragma unroll
          for (int m = 0; m < RS; ++m) {
            const uint2 o = row[m];  // the same address across the half-wave: a broadcast
            rank += (m < n_ent && better(__uint_as_float(o.x), (int)o.y, __uint_as_float(mine.x), (int)mine.y)) ? 1 : 0;
          }
          __builtin_amdgcn_wave_barrier();  // every lane has read before any lane writes
          if (l < n_ent && rank < kk) row[rank] = mine;
          if (l == 0 && c > 0) cnt_s[hw + 16 * i] = 0;
        }
        if (tid == 0) wait_s[(round + 1) & 1] = 0;
      }
      again = wait_s[round & 1] != 0;
      ++round;
      __syncthreads();
    } while (again);
  }
  }  // tiles

  if (TOPK) {
    // the lists of this range (unordered; unused slots hold -inf / INT_MAX): joined by topk_merge_kernel
    for (int e = tid; e < TM * a.topk; e += 512) {
      const int row = e / a.topk, j = e - row * a.topk;
      if (m0 + row < a.M) {
        const int64_t o = ((((int64_t)group * a.M + m0 + row) * a.ranges) + range) * a.topk + j;
        a.part_val[o] = __uint_as_float(list[row * RS + j].x);
        a.part_idx[o] = (int)list[row * RS + j].y;
      }
    }
  }
}

// One wavefront per query: the ranges * k (score, index) pairs of the row, k rounds of arg-best.
__global__ __launch_bounds__(64) void topk_merge_kernel(const float* __restrict__ part_val, const int32_t* __restrict__ part_idx,
                                                        const int cands, const int k, int32_t* __restrict__ out_idx,
                                                        float* __restrict__ out_val) {
  constexpr int PER = 64;  // pairs per lane: at most 4096 pairs per row (checked at launch)
  const int lane = threadIdx.x;
  const int64_t row = blockIdx.x;
  const float NEG = -__builtin_inff();
  float v[PER];
  int id[PER];
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const int c = e * 64 + lane;
    v[e] = c < cands ? part_val[row * cands + c] : NEG;
    id[e] = c < cands ? part_idx[row * cands + c] : 0x7fffffff;
  }
  for (int r = 0; r < k; ++r) {
    float bv = NEG;
    int bi = 0x7fffffff;
#pragma unroll
    for (int e = 0; e < PER; ++e)
      if (e * 64 < cands && better(v[e], id[e], bv, bi)) {
        bv = v[e];
        bi = id[e];
      }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const float ov = __shfl_xor(bv, off);
      const int oi = __shfl_xor(bi, off);
      if (better(ov, oi, bv, bi)) {
        bv = ov;
        bi = oi;
      }
    }
    // the winner leaves the set (indices of real pairs are distinct)
#pragma unroll
    for (int e = 0; e < PER; ++e)
      if (id[e] == bi && bi != 0x7fffffff) {
        v[e] = NEG;
        id[e] = 0x7fffffff;
      }
    if (lane == 0) {
      out_idx[row * k + r] = bi == 0x7fffffff ? -1 : bi;
      if (out_val != nullptr) out_val[row * k + r] = bv;
    }
  }
}

// Ranges of code tiles per query block for the fused top-k: about one workgroup per compute unit in all
// (the kernel's LDS admits one), every range at least one tile; from 8 ranges on the count is kept a multiple
// of 8 so that every XCD can take whole ranges (xcd_split = ranges per XCD, 0: no such split).
int plan_ranges(int64_t tiles_n, int nqb, int* xcd_split) {
  int64_t r = device_cu_count() / nqb;
  if (r > tiles_n) r = tiles_n;
  if (r > 256) r = 256;
  if (r < 1) r = 1;
  *xcd_split = 0;
  if (r >= 8) {
    r -= r % 8;
    *xcd_split = (int)(r / 8);
  }
  return (int)r;
}

template <int BITS, bool PROD, int TM, int TN>
hipError_t launch_tile(const Bf3Args& a0, int n_groups, hipStream_t s) {
  using C = Cfg<BITS, PROD, TM, TN>;
  if (!C::FITS) return hipErrorInvalidValue;
  if (a0.topk > 0) {
    Bf3Args a = a0;
    a.groups = n_groups;
    a.tiles_n = (int)((a.n + TN - 1) / TN);
    a.qblocks = (a.M + TM - 1) / TM;
    a.ranges = plan_ranges(a.tiles_n, a.qblocks * n_groups, &a.xcd_split);
    static LdsLimit lds_limit;  // per instantiation: the limit is raised once per device
    if (const hipError_t e = raise_lds_limit(lds_limit, reinterpret_cast<const void*>(&score_bf3_kernel<BITS, PROD, TM, TN, true>), C::LDS_BYTES_TOPK); e != hipSuccess) return e;
    hipLaunchKernelGGL((score_bf3_kernel<BITS, PROD, TM, TN, true>), dim3((unsigned)(a.qblocks * n_groups * a.ranges)), dim3(512),
                       C::LDS_BYTES_TOPK, s, a);
    return hipGetLastError();
  }
  static LdsLimit lds_limit;  // per instantiation: the limit is raised once per device
  if (const hipError_t e = raise_lds_limit(lds_limit, reinterpret_cast<const void*>(&score_bf3_kernel<BITS, PROD, TM, TN, false>), C::LDS_BYTES); e != hipSuccess) return e;
  Bf3Args a = a0;
  a.tiles_n = (int)((a.n + TN - 1) / TN);
  const int64_t total = (int64_t)a.tiles_n * ((a.M + TM - 1) / TM);
  if (total > 0x7ffffff0) return hipErrorInvalidValue;
  a.xcd_split = (a.transposed || (a.M + TM - 1) / TM > 4) ? 1 : 0;
  const dim3 grid = a.xcd_split ? dim3((unsigned)((total + 7) / 8 * 8), 1, n_groups)
                                : dim3((unsigned)a.tiles_n, (unsigned)((a.M + TM - 1) / TM), n_groups);
  hipLaunchKernelGGL((score_bf3_kernel<BITS, PROD, TM, TN, false>), grid, dim3(512), C::LDS_BYTES, s, a);
  return hipGetLastError();
}

// 256 queries per tile halve the LDS reads per MFMA (a wavefront's sub-tiles share fragments), which is what
// bounds the 128-row tile; the accumulators of two segments do not fit that shape
// Two-stage codes with more than one index bit need four code-side operands (three centroid pieces and the
// signs): 128 codes per tile, so that two buffers still fit.
template <int BITS, bool PROD>
hipError_t launch_one(const Bf3Args& a, int n_groups, hipStream_t s) {
  if (PROD && BITS >= 2) return launch_tile<BITS, PROD, 128, 128>(a, n_groups, s);
  if (!PROD && a.M > 128) return launch_tile<BITS, PROD, PROD ? 128 : 256, 256>(a, n_groups, s);
  return launch_tile<BITS, PROD, 128, (PROD && BITS >= 2) ? 128 : 256>(a, n_groups, s);
}

}  // namespace

// what the kernel takes: both LDS buffers must fit, and the 1-bit codebook must be +-c
bool score_bf3_applicable(int bits, bool prod, int d, int64_t n, int n_groups, int q_per_group, const Codebook& cb) {
  if (d % 32 != 0 || n <= 0 || q_per_group <= 0 || n_groups > 65535 || (q_per_group + 127) / 128 > 65535) return false;
  if (bits == 0) return prod;
  if (bits == 1) return cb.c[0] == -cb.c[1];
  return bits <= 4;
}

// the tile launch_one picks, and with it the fused top-k's ranges
int score_bf3_topk_ranges(int bits, bool prod, int64_t n, int n_groups, int q_per_group, int topk) {
  if (topk < 1 || topk > KL || n <= 0 || n_groups <= 0 || q_per_group <= 0) return 0;
  const int tm = (!prod && q_per_group > 128) ? 256 : 128, tn = (prod && bits >= 2) ? 128 : 256;
  const int64_t nqb = (int64_t)((q_per_group + tm - 1) / tm) * n_groups;
  if (nqb > 0x7fffffff / 256) return 0;
  int xs;
  return plan_ranges((n + tn - 1) / tn, (int)nqb, &xs);
}

hipError_t launch_topk_merge(const float* part_val, const int32_t* part_idx, int64_t rows, int ranges, int k,
                             int32_t* out_idx, float* out_val, hipStream_t s) {
  if (rows == 0) return hipSuccess;
  if (ranges < 1 || k < 1 || k > 64 || (int64_t)ranges * k > 4096 || rows > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(topk_merge_kernel, dim3((unsigned)rows), dim3(64), 0, s, part_val, part_idx, ranges * k, k, out_idx, out_val);
  return hipGetLastError();
}

hipError_t launch_score_bf3(int bits, bool prod, const float* qr, const float* qs, int q_per_group, int d,
                            const uint32_t* idx, const uint32_t* qjl, const float* gamma, const float* norm, int64_t n,
                            int n_groups, float* out, int64_t ldo, bool transposed, float kappa, const Codebook& cb,
                            hipStream_t s, int topk, float* part_val, int32_t* part_idx) {
  Bf3Args a;
  std::memset(&a, 0, sizeof(a));
  if (topk > 0 && (transposed || topk > KL || part_val == nullptr || part_idx == nullptr)) return hipErrorInvalidValue;
  a.topk = topk; a.part_val = part_val; a.part_idx = part_idx;
  a.transposed = transposed ? 1 : 0;
  a.qr = qr; a.qs = qs; a.M = q_per_group; a.d = d; a.idx = idx; a.qjl = qjl; a.gamma = gamma; a.norm = norm;
  a.n = n; a.out = out; a.ldo = ldo; a.kappa = kappa; a.cb = cb;
  switch (bits * 2 + (prod ? 1 : 0)) {
    case 1: return launch_one<0, true>(a, n_groups, s);
    case 2: return launch_one<1, false>(a, n_groups, s);
    case 3: return launch_one<1, true>(a, n_groups, s);
    case 4: return launch_one<2, false>(a, n_groups, s);
    case 5: return launch_one<2, true>(a, n_groups, s);
    case 6: return launch_one<3, false>(a, n_groups, s);
    case 7: return launch_one<3, true>(a, n_groups, s);
    case 8: return launch_one<4, false>(a, n_groups, s);
    case 9: return launch_one<4, true>(a, n_groups, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace tq
