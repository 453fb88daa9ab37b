// Quant_mse / Quant_prod (Alg. 1 / Alg. 2) at d = 128 for batches of bf16 vectors beyond what one round of the
// small-batch kernel covers, on the bf16 matrix cores (exact bf16 pieces of the fp32 factors, see tq_bf3.h): the
// rotation to fp32 accuracy, the sketch as far as its signs need.
//
//   stage 1   y^T = Pi x^T.  A bf16 input IS a single piece, so the rotation takes three piece products
//             (x times the three pieces of Pi).  The vector is the COLUMN of the MFMA: a lane loads 8
//             consecutive bf16 of its vector's row from HBM and that register is the B operand as it
//             stands; the A operand is a piece of Pi, resident in LDS for the life of the workgroup.
//   decision  the accumulator tile holds 16 coordinates of one vector per lane: scale by 1 / ||x||, nearest
//             centroid, packing, residual e = y - c[idx] in place (quantise_tile), gamma = ||e||.
//   stage 2   u^T = (S Pi^T) e^T, of which only the signs are kept.  The residual registers, split into their
//             two leading pieces, are directly the B operand (the order in which they enumerate the
//             contraction index is a fixed permutation inside every run of 16, which the LDS image of
//             S Pi^T follows).  S Pi^T is held as its two leading pieces as well, and the three products of
//             combined weight >= 2^-9 are taken: what is left out is 2^-17.8 of a term (root mean square), about
//             5e-7 |S_j| |e| in u, against the 1e-5 |S_j| |e| inside which a sign may differ from the exact one.
//   LDS       three pieces of Pi and two of S Pi^T, 128 x 128 bf16 each, are exactly the 160 KB of a compute
//             unit: rows are stored without padding, the 16-byte chunks of a row rotated by the row number
//             (conflict-free 16-byte reads along a column of chunks).
//
// Workgroup = 8 wavefronts (two per SIMD), a wavefront takes 32 vectors per block of 256.  Four wavefronts of
// 64 vectors (VT = 2: the register file of a SIMD to one wavefront, every LDS read of an A operand feeding two
// MFMAs) are 13-19 % slower: nothing runs on a SIMD while its one wavefront is in the decision stage's
// dependent chains or waits for LDS.
#include <type_traits>

#include "tq_bf3.h"
#include "tq_d128_tile.h"

namespace tq {

namespace {

constexpr int MAT_ELEMS = 128 * 128;  // one piece of one matrix
constexpr int PI_ELEMS = 3 * MAT_ELEMS;
constexpr int W_ELEMS = 2 * MAT_ELEMS;
constexpr int RING = 4;  // A operands in flight

// element offset of column col (a multiple of 4) of row `row` inside a piece: chunk (col / 8) xor (row % 16)
__device__ __forceinline__ int lds_at(int row, int col) { return row * 128 + ((((col >> 3) ^ row) & 15) << 3) + (col & 7); }

struct Q128Args {
  const void* X;  // bf16, or fp32 in the F32 instantiations
  int64_t ldx;
  int64_t n;
  const float* Pi;
  const float* SPiT;
  const u32x4* image;  // nullable: the LDS image below, made ahead of time by q128_image_kernel
  uint32_t* idx;
  uint32_t* qjl;
  float* gamma;
  float* norm;  // nullable: no normalisation then
  Codebook cb;
  // two instances over a split of the rotated coordinates (MIXED, Sec. 4.3): coordinate groups (= output tiles)
  // [0, gs_hi) are quantised with BITS + 1 bits and cb_hi, each instance normalised by the norm of its own rotated
  // coordinates; idx rows then hold 4 BITS + gs_hi words, gamma and norm two floats per vector (hi, lo)
  int gs_hi;
  Codebook cb_hi;
};

// sum of the squares of two bf16 values added to acc: one two-element dot product with fp32 accumulation
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float square_pair(uint32_t w, float acc) {
  const bf16x2_t v = __builtin_bit_cast(bf16x2_t, w);
  return __builtin_amdgcn_fdot2_f32_bf16(v, v, acc, false);
}

// position of column j inside its run of 16 in the image of S Pi^T: the two middle groups of four change
// places (see stage 2)
__device__ __forceinline__ int w_col(int j) { return (j & ~12) | ((j & 4) << 1) | ((j & 8) >> 1); }

// The kernel's parameter image, by 256 threads: three pieces of Pi at dst, two of S Pi^T (columns permuted) behind
// them, each [row][128] with the chunk rotation of lds_at.  dst is LDS in the quantisation kernel and device
// memory in q128_image_kernel.
__device__ __forceinline__ void q128_split_matrices(const float* Pi, const float* SPiT, unsigned short* dst, int tid) {
  // rows [row0, row0 + 64) of a 128 x 128 fp32 matrix -> its leading `pieces` pieces; 8 x 16 bytes per thread
  auto split_rows = [&](const f32x4 (&v)[8], unsigned short* out, int row0, int pieces, bool permute) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int e = (i * 256 + tid) * 4;
      const int row = row0 + (e >> 7), j = e & 127;
      uint32_t lo[3], hi[3];
      split3_pair(f32x2{v[i][0], v[i][1]}, lo[0], lo[1], lo[2]);
      split3_pair(f32x2{v[i][2], v[i][3]}, hi[0], hi[1], hi[2]);
      const int at = lds_at(row, permute ? w_col(j) : j);
#pragma unroll
      for (int pc = 0; pc < 3; ++pc)
        if (pc < pieces) *reinterpret_cast<uint2*>(out + pc * MAT_ELEMS + at) = make_uint2(lo[pc], hi[pc]);
    }
  };
  auto fetch64 = [&](const float* src, f32x4 (&v)[8]) {
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = *reinterpret_cast<const f32x4*>(src + (i * 256 + tid) * 4);
  };
  f32x4 lo[8], hi[8];
  fetch64(Pi, lo);
  fetch64(Pi + 64 * 128, hi);
  split_rows(lo, dst, 0, 3, false);
  split_rows(hi, dst, 64, 3, false);
  if (SPiT != nullptr) {
    fetch64(SPiT, lo);
    fetch64(SPiT + 64 * 128, hi);
    split_rows(lo, dst + PI_ELEMS, 0, 2, true);
    split_rows(hi, dst + PI_ELEMS, 64, 2, true);
  }
}

// one workgroup of 256 threads: the image in device memory, (PI_ELEMS + W_ELEMS) * 2 bytes
__global__ __launch_bounds__(256) void q128_image_kernel(const float* Pi, const float* SPiT, unsigned short* image) {
  q128_split_matrices(Pi, SPiT, image, threadIdx.x);
}

// VT = vector tiles (of 32) per wavefront: 2 = four wavefronts of 64 vectors (one per SIMD, every LDS read of an A
// operand feeds two MFMAs), 1 = eight wavefronts of 32 vectors (two per SIMD: while one is in its decision stage or
// waits for LDS, the other issues MFMAs).
//
// F32: the vectors are fp32.  A lane's 8 values of a step are two 16-byte loads, split into their two leading
// pieces (x1 + x2 = x up to 2^-17 |x|), and the rotation takes the five piece products of weight >= 2^-16 that two
// pieces of x have with three of Pi: every A operand read of the two leading pieces of Pi feeds two MFMAs.
template <int BITS, bool PROD, bool MIXED, int VT, bool F32 = false>
__global__ __launch_bounds__(512 / VT) void quant128_bf3_kernel(const Q128Args a) {
  constexpr int NT = 512 / VT;  // threads
  constexpr int NB = (BITS > 0 ? BITS : 1) + (MIXED ? 1 : 0);  // plane words per tile, at most
  constexpr int BH = BITS < 4 ? BITS + 1 : 4;                  // bits of instance hi
  extern __shared__ __attribute__((aligned(16))) unsigned short lds_s[];
  unsigned short* const Pi_s = lds_s;            // [piece][row j][128], see lds_at
  unsigned short* const W_s = lds_s + PI_ELEMS;  // [piece][row j'][128], columns permuted
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int vi = lane & 31, g = lane >> 5;

  if (a.image != nullptr) {
    // a straight copy, 16 bytes per thread and step: 24 steps for Pi, 16 for S Pi^T
    constexpr int STEPS = (PI_ELEMS + (PROD ? W_ELEMS : 0)) * 2 / (NT * 16);
    u32x4* const dst = reinterpret_cast<u32x4*>(lds_s);
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      u32x4 v[STEPS / 2];
#pragma unroll
      for (int i = 0; i < STEPS / 2; ++i) v[i] = a.image[(half * (STEPS / 2) + i) * NT + tid];
#pragma unroll
      for (int i = 0; i < STEPS / 2; ++i) dst[(half * (STEPS / 2) + i) * NT + tid] = v[i];
    }
  } else if (tid < 256) {
    q128_split_matrices(a.Pi, PROD ? a.SPiT : nullptr, lds_s, tid);
  }
  __syncthreads();

  const int64_t blocks = (a.n + 255) / 256;
  const bool normalise = !MIXED && a.norm != nullptr;
  constexpr int ESZ = F32 ? 4 : 2;
  u32x4 xop[VT][8];                   // the B operands of stage 1 (F32: piece 1 of x)
  u32x4 xop2[F32 ? VT : 1][8];        // F32: piece 2
  u32x4 xraw[F32 ? VT : 1][8][2];     // F32: the fp32 values as loaded
  auto x_row = [&](int64_t blk, int nt) {  // this lane's 8 values of step 0
    const int64_t v = blk * 256 + wave * (32 * VT) + 32 * nt + vi;
    return static_cast<const char*>(a.X) + ((v < a.n ? v : a.n - 1) * a.ldx + 8 * g) * ESZ;  // clamped: such vectors are not stored
  };
  auto load_x = [&](const char* src, int nt, int s) {  // the 8 values of step s
    if constexpr (F32) {
      xraw[nt][s][0] = *reinterpret_cast<const u32x4*>(src + 64 * s);
      xraw[nt][s][1] = *reinterpret_cast<const u32x4*>(src + 64 * s + 16);
    } else {
      xop[nt][s] = *reinterpret_cast<const u32x4*>(src + 32 * s);
    }
  };
#pragma unroll
  for (int nt = 0; nt < VT; ++nt) {
    const char* src = x_row(blockIdx.x, nt);
#pragma unroll
    for (int s = 0; s < 8; ++s) load_x(src, nt, s);
  }

  for (int64_t blk = blockIdx.x; blk < blocks; blk += gridDim.x) {
    // ---- norms: a lane and its partner in the other half-wave hold one vector between them --------------
    float nu[VT], inv[VT];
#pragma unroll
    for (int nt = 0; nt < VT; ++nt) nu[nt] = inv[nt] = 1.f;
    if (normalise) {
#pragma unroll
      for (int nt = 0; nt < VT; ++nt) {
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          if constexpr (F32) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
              const f32x4 v = __builtin_bit_cast(f32x4, xraw[nt][s][h]);
              s0 = fmaf(v[0], v[0], s0);
              s1 = fmaf(v[1], v[1], s1);
              s0 = fmaf(v[2], v[2], s0);
              s1 = fmaf(v[3], v[3], s1);
            }
          } else {
            s0 = square_pair(xop[nt][s][0], s0);
            s1 = square_pair(xop[nt][s][1], s1);
            s0 = square_pair(xop[nt][s][2], s0);
            s1 = square_pair(xop[nt][s][3], s1);
          }
        }
        nu[nt] = sqrtf(add_across_halves(s0 + s1));
        inv[nt] = nu[nt] > 0.f ? 1.f / nu[nt] : 0.f;
      }
    }

    if constexpr (F32) {
      // the two leading pieces of the vectors: word j of a step's operand holds values 2 j and 2 j + 1
#pragma unroll
      for (int nt = 0; nt < VT; ++nt)
#pragma unroll
        for (int s = 0; s < 8; ++s)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const f32x4 v = __builtin_bit_cast(f32x4, xraw[nt][s][j >> 1]);
            uint32_t w1, w2;
            split2_pair(f32x2{v[2 * (j & 1)], v[2 * (j & 1) + 1]}, w1, w2);
            xop[nt][s][j] = w1;
            xop2[nt][s][j] = w2;
          }
    }

    // ---- stage 1: y^T = Pi x^T, three piece products (F32: five) ----------------------------------------
    // (the first product of every accumulator takes a zero C operand: nothing is cleared)
    floatx16 acc[VT][4];
    const floatx16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    {
      // the A operands travel through a ring of RING registers, read RING MFMA pairs ahead of their use: left to
      // itself the compiler reuses two registers and every group of MFMAs waits for a full LDS round trip
      auto pi_piece = [&](int i) {  // read i of 96: step i / 12, pieces 2, 1, 0 (smallest products first), tile i % 4
        return *reinterpret_cast<const bf16x8*>(Pi_s + (2 - (i >> 2) % 3) * MAT_ELEMS + lds_at(32 * (i & 3) + vi, 16 * (i / 12) + 8 * g));
      };
      bf16x8 ring[RING];
#pragma unroll
      for (int i = 0; i < RING; ++i) ring[i] = pi_piece(i);
#pragma unroll
      for (int i = 0; i < 96; ++i) {
        const int s = i / 12, t = i & 3;
#pragma unroll
        for (int nt = 0; nt < VT; ++nt)
          acc[nt][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[i % RING], *reinterpret_cast<const bf16x8*>(&xop[nt][s]),
                                                               i < 4 ? zero16 : acc[nt][t], 0, 0, 0);
        if constexpr (F32) {
          if ((i >> 2) % 3 != 0) {  // pieces 1 and 0 of Pi also meet piece 2 of x
#pragma unroll
            for (int nt = 0; nt < VT; ++nt)
              acc[nt][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[i % RING], *reinterpret_cast<const bf16x8*>(&xop2[nt][s]),
                                                                   acc[nt][t], 0, 0, 0);
          }
        }
        if (i + RING < 96) ring[i % RING] = pi_piece(i + RING);
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    // ---- decision: indices, packing, residual in place; the residual's pieces ---------------------------
    // register 4 k + r of tile t holds coordinate j = 32 t + 8 k + 4 g + r of the lane's vector
    uint32_t word[VT][4][NB];
    float g2[VT] = {}, g2h[VT] = {}, nuh[VT] = {};  // MIXED: g2 / nu belong to instance lo
    u32x4 rp[2][VT][8];  // [piece][nt][step of stage 2]
    const int gs = MIXED ? a.gs_hi : 0;
    float inv_hi[VT] = {};
#pragma unroll
    for (int nt = 0; nt < VT; ++nt) {
      if (MIXED) {
        // the norms of the two instances from the rotated coordinates (the rotation is block diagonal)
        float s_hi = 0.f, s_lo = 0.f;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          float s0 = 0.f, s1 = 0.f;
#pragma unroll
          for (int r = 0; r < 16; r += 2) {
            s0 = fmaf(acc[nt][t][r], acc[nt][t][r], s0);
            s1 = fmaf(acc[nt][t][r + 1], acc[nt][t][r + 1], s1);
          }
          s_hi += t < gs ? s0 + s1 : 0.f;
          s_lo += t < gs ? 0.f : s0 + s1;
        }
        nuh[nt] = sqrtf(add_across_halves(s_hi));
        nu[nt] = sqrtf(add_across_halves(s_lo));
        inv_hi[nt] = nuh[nt] > 0.f ? 1.f / nuh[nt] : 0.f;
        inv[nt] = nu[nt] > 0.f ? 1.f / nu[nt] : 0.f;
      }
    }
    {
      // one tile; nt and t arrive as types so that every register index below is a constant whatever the compiler
      // decides about unrolling (left as loops, the two-instance body with 15 compares was not unrolled and its
      // arrays went to scratch memory)
      auto tile = [&](auto nt_c, auto t_c) {
        constexpr int nt = decltype(nt_c)::value, t = decltype(t_c)::value;
        uint32_t wd[4] = {0u, 0u, 0u, 0u};
        if (MIXED && t < gs)  // uniform
          g2h[nt] += quantise_tile_best<BH>(acc[nt][t], inv_hi[nt], a.cb_hi, g, wd);
        else
          g2[nt] += quantise_tile_best<BITS>(acc[nt][t], inv[nt], a.cb, g, wd);
#pragma unroll
        for (int pl = 0; pl < NB; ++pl) word[nt][t][pl] = wd[pl];
        if (PROD) {
#pragma unroll
          for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              uint32_t w1, w2;
              split2_pair(f32x2{acc[nt][t][8 * p + 2 * e], acc[nt][t][8 * p + 2 * e + 1]}, w1, w2);
              rp[0][nt][2 * t + p][e] = w1;
              rp[1][nt][2 * t + p][e] = w2;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
      };
      using I0 = std::integral_constant<int, 0>;
      using I1 = std::integral_constant<int, 1>;
      using I2 = std::integral_constant<int, 2>;
      using I3 = std::integral_constant<int, 3>;
      tile(I0{}, I0{}); tile(I0{}, I1{}); tile(I0{}, I2{}); tile(I0{}, I3{});
      if constexpr (VT == 2) {
        tile(I1{}, I0{}); tile(I1{}, I1{}); tile(I1{}, I2{}); tile(I1{}, I3{});
      }
    }

    // the vector this lane stores for.  VT = 2: tile nt = g (each half-wave writes one tile's rows); VT = 1: the one
    // tile, by the lower half-wave (both halves hold the merged words)
    const int64_t v_mine = VT == 2 ? blk * 256 + wave * 64 + 32 * g + vi : blk * 256 + wave * 32 + vi;
    const bool storing = v_mine < a.n && (VT == 2 || g == 0);
    constexpr int HI = VT - 1;  // the tile of the upper half-wave
    // the next block's vectors are fetched while this block is finished: spread over the first pass of stage 2
    const char* const next_x[2] = {x_row(blk + gridDim.x, 0), x_row(blk + gridDim.x, HI)};
    if (!PROD) {
#pragma unroll
      for (int nt = 0; nt < VT; ++nt)
#pragma unroll
        for (int s = 0; s < 8; ++s) load_x(next_x[nt], nt, s);
    }

    // ---- the codes of Alg. 1: lane (vi, g) writes the row of vector 32 g + vi ----------------------------
    const uint32_t mine = VT == 2 ? 0u - (uint32_t)g : 0u;  // all ones in the half-wave that stores tile nt = 1
    if (storing) {
      // word[g][t][pl], selected with a mask (an indexed array would live in scratch memory)
      if (MIXED) {
        uint32_t* dst = a.idx + v_mine * (4 * BITS + gs);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const bool thi = t < gs;
#pragma unroll
          for (int pl = 0; pl < BITS + 1; ++pl)
            if (pl < BITS || thi) dst[pl] = word[0][t][pl] ^ ((word[0][t][pl] ^ word[HI][t][pl]) & mine);
          dst += thi ? BITS + 1 : BITS;
        }
        *reinterpret_cast<float2*>(a.norm + 2 * v_mine) = make_float2(g ? nuh[HI] : nuh[0], g ? nu[HI] : nu[0]);
      } else {
        if (BITS > 0) {
          uint32_t* dst = a.idx + v_mine * (4 * BITS);
          uint32_t row[4 * NB];
#pragma unroll
          for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int pl = 0; pl < BITS; ++pl) row[t * BITS + pl] = word[0][t][pl] ^ ((word[0][t][pl] ^ word[HI][t][pl]) & mine);
#pragma unroll
          for (int q = 0; q < BITS; ++q)
            *reinterpret_cast<u32x4*>(dst + 4 * q) = u32x4{row[4 * q], row[4 * q + 1], row[4 * q + 2], row[4 * q + 3]};
        }
        if (normalise) a.norm[v_mine] = g ? nu[HI] : nu[0];
      }
    }

    if (PROD) {
      // ---- stage 2: u^T = (S Pi^T) e^T, three piece products, one half of the output coordinates at a time ----
      uint32_t sw[VT][4];  // [nt][sign word]
#pragma unroll
      for (int pass = 0; pass < 2; ++pass) {
        floatx16 u[VT][2];
        {
          auto w_piece = [&](int i) {  // read i of 32: step i / 4, pieces 1, 0, tile i % 2
            return *reinterpret_cast<const bf16x8*>(W_s + (1 - ((i >> 1) & 1)) * MAT_ELEMS +
                                                    lds_at(64 * pass + 32 * (i & 1) + vi, 16 * (i >> 2) + 8 * g));
          };
          bf16x8 ring[RING];
#pragma unroll
          for (int i = 0; i < RING; ++i) ring[i] = w_piece(i);
#pragma unroll
          for (int i = 0; i < 32; ++i) {
            const int s = i >> 2, pa = 1 - ((i >> 1) & 1), mt = i & 1;
#pragma unroll
            for (int pb = 1 - pa; pb >= 0; --pb)
#pragma unroll
              for (int nt = 0; nt < VT; ++nt)
                u[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[i % RING], *reinterpret_cast<const bf16x8*>(&rp[pb][nt][s]),
                                                                    i < 2 ? zero16 : u[nt][mt], 0, 0, 0);
            if (i + RING < 32) ring[i % RING] = w_piece(i + RING);
            // the next block's vectors: all sixteen loads during the first pass
            if (pass == 0 && (i & 1) && (VT == 2 || !(i & 2)))
              load_x(next_x[(i >> 1) & 1], (i >> 1) & HI, s);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        // signs: register 4 k + r of tile mt is coordinate 64 pass + 32 mt + 8 k + 4 g + r.  The bit of Def. 1 is
        // "u >= 0", the complement of the fp32 sign bit: a sum of products accumulated from +0 is never -0 (exact
        // cancellation rounds to +0), so the sign bits are shifted in, one instruction each, and inverted at the end.
#pragma unroll
        for (int nt = 0; nt < VT; ++nt)
#pragma unroll
          for (int mt = 0; mt < 2; ++mt) {
            uint32_t nib[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              nib[k] = 0u;
#pragma unroll
              for (int r = 3; r >= 0; --r) nib[k] = __builtin_amdgcn_alignbit(nib[k], __float_as_uint(u[nt][mt][4 * k + r]), 31);
            }
            const uint32_t w = ((nib[0] | (nib[1] << 8) | (nib[2] << 16) | (nib[3] << 24)) ^ 0x0f0f0f0fu) << (4 * g);
            sw[nt][2 * pass + mt] = or_across_halves(w);
          }
      }
      // (exchanges between the half-waves stay outside the guarded stores: every lane takes part)
#pragma unroll
      for (int nt = 0; nt < VT; ++nt) {
        g2[nt] = add_across_halves(g2[nt]);
        if (MIXED) g2h[nt] = add_across_halves(g2h[nt]);
      }
      if (storing) {
        *reinterpret_cast<u32x4*>(a.qjl + v_mine * 4) =
            g ? u32x4{sw[HI][0], sw[HI][1], sw[HI][2], sw[HI][3]} : u32x4{sw[0][0], sw[0][1], sw[0][2], sw[0][3]};
        if (MIXED) {
          *reinterpret_cast<float2*>(a.gamma + 2 * v_mine) = make_float2(sqrtf(g ? g2h[HI] : g2h[0]), sqrtf(g ? g2[HI] : g2[0]));
        } else {
          a.gamma[v_mine] = sqrtf(g ? g2[HI] : g2[0]);
        }
      }
    }
  }
}

template <int BITS, bool PROD, bool MIXED, int VT, bool F32>
hipError_t launch_vt(const Q128Args& a, hipStream_t s) {
  constexpr int lds = (PI_ELEMS + (PROD ? W_ELEMS : 0)) * 2;
  static LdsLimit lds_limit;  // per instantiation: the limit is raised once per device
  if (const hipError_t e = raise_lds_limit(lds_limit, reinterpret_cast<const void*>(&quant128_bf3_kernel<BITS, PROD, MIXED, VT, F32>), lds); e != hipSuccess) return e;
  const int64_t blocks = (a.n + 255) / 256, cus = device_cu_count();  // one workgroup per compute unit
  hipLaunchKernelGGL((quant128_bf3_kernel<BITS, PROD, MIXED, VT, F32>), dim3((unsigned)(blocks < cus ? blocks : cus)), dim3(512 / VT), lds, s, a);
  return hipGetLastError();
}

// eight wavefronts of 32 vectors: measured against four of 64 (VT = 2) on the same box, 524288 vectors, 2 + 1 bits:
// 109 against 125 us; 3 + 1 bits: 122 against 150; two instances: 105 against 124; 131072 vectors: 33 against 38
template <int BITS, bool PROD, bool MIXED>
hipError_t launch_one(const Q128Args& a, bool f32, hipStream_t s) {
  if constexpr (!MIXED) {
    if (f32) return launch_vt<BITS, PROD, MIXED, 1, true>(a, s);
  }
  return launch_vt<BITS, PROD, MIXED, 1, false>(a, s);
}

}  // namespace

// bf16 rows of 128 values (fp32 rows too where there is one instance), 16-byte aligned with a row stride that keeps
// them so; symmetric tables
bool quant128_bf3_applicable(int bits, bool prod, bool f32, const void* X, int64_t ldx, const Codebook& cb, const Codebook* cb_hi) {
  if (f32 && cb_hi != nullptr) return false;
  if (bits < 0 || bits > (cb_hi != nullptr ? 3 : 4) || (bits == 0 && !prod && cb_hi == nullptr)) return false;
  // from 3 bits on the decision is taken on |y|: tables symmetric about zero (what tq_build_codebook produces)
  if (!codebook_symmetric(cb, bits) || (cb_hi != nullptr && !codebook_symmetric(*cb_hi, bits + 1))) return false;
  return (reinterpret_cast<uintptr_t>(X) & 15u) == 0 && ldx % (f32 ? 4 : 8) == 0;
}

// gs_hi > 0: two instances (cb_hi with bits + 1 bits for the first gs_hi coordinate groups); norm is required then
hipError_t launch_quant128_bf3(int bits, bool prod, bool f32, const void* X, int64_t ldx, int64_t n, const float* Pi,
                               const float* SPiT, uint32_t* idx, uint32_t* qjl, float* gamma, float* norm,
                               const Codebook& cb, int gs_hi, const Codebook& cb_hi, const void* image, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  if (gs_hi < 0 || gs_hi > 3 || (gs_hi > 0 && (f32 || bits > 3 || cb_hi.bits != bits + 1 || norm == nullptr))) return hipErrorInvalidValue;
  if (!codebook_symmetric(cb, bits) || (gs_hi > 0 && !codebook_symmetric(cb_hi, bits + 1))) return hipErrorInvalidValue;
  Q128Args a;
  a.X = X; a.ldx = ldx; a.n = n; a.Pi = Pi; a.SPiT = SPiT; a.idx = idx; a.qjl = qjl;
  a.image = static_cast<const u32x4*>(image);
  a.gamma = gamma; a.norm = norm; a.cb = cb; a.gs_hi = gs_hi; a.cb_hi = cb_hi;
  if (gs_hi > 0) {
    switch (bits * 2 + (prod ? 1 : 0)) {
      case 0: return launch_one<0, false, true>(a, f32, s);
      case 1: return launch_one<0, true, true>(a, f32, s);
      case 2: return launch_one<1, false, true>(a, f32, s);
      case 3: return launch_one<1, true, true>(a, f32, s);
      case 4: return launch_one<2, false, true>(a, f32, s);
      case 5: return launch_one<2, true, true>(a, f32, s);
      case 6: return launch_one<3, false, true>(a, f32, s);
      case 7: return launch_one<3, true, true>(a, f32, s);
      default: return hipErrorInvalidValue;
    }
  }
  switch (bits * 2 + (prod ? 1 : 0)) {
    case 1: return launch_one<0, true, false>(a, f32, s);
    case 2: return launch_one<1, false, false>(a, f32, s);
    case 3: return launch_one<1, true, false>(a, f32, s);
    case 4: return launch_one<2, false, false>(a, f32, s);
    case 5: return launch_one<2, true, false>(a, f32, s);
    case 6: return launch_one<3, false, false>(a, f32, s);
    case 7: return launch_one<3, true, false>(a, f32, s);
    case 8: return launch_one<4, false, false>(a, f32, s);
    case 9: return launch_one<4, true, false>(a, f32, s);
    default: return hipErrorInvalidValue;
  }
}

size_t quant128_bf3_image_bytes() { return (size_t)(PI_ELEMS + W_ELEMS) * 2; }

// SPiT may be null (no sketch): the second part of the image is left alone then
hipError_t launch_quant128_bf3_image(const float* Pi, const float* SPiT, void* image, hipStream_t s) {
  hipLaunchKernelGGL(q128_image_kernel, dim3(1), dim3(256), 0, s, Pi, SPiT, static_cast<unsigned short*>(image));
  return hipGetLastError();
}

}  // namespace tq
