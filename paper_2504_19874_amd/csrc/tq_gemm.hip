// Generic fp32 MFMA contraction for gfx950 with on-the-fly operand decoding
// and fused quantisation epilogues.  See tq_internal.h for what it computes.
//
// Tiling.  One workgroup = 256 threads = 4 wavefronts arranged 2 x 2; the
// workgroup owns a 128 (rows m) x 128 (vectors i) block of D, each wavefront
// a 64 x 64 block = 2 x 2 tiles of v_mfma_f32_32x32x2_f32 (64 accumulator
// registers).  K advances 32 at a time through LDS; both operand tiles are
// stored [row][k] with a row stride of 36 floats, so that a lane's 16-byte
// read of four consecutive k lands in banks 4*row + const: conflict free.
//
// Operand layout of v_mfma_f32_32x32x2_f32 (A is 32x2, B is 2x32, D is 32x32):
//   A[i][k] sits in lane i + 32k, B[k][j] in lane j + 32k,
//   D[i][j] in lane j + 32*((i/4)%2), register 4*(i/8) + i%4.
// The contraction index may be visited in any order as long as A and B agree.
// Here lane half h = lane/32 reads k = 8s + 4h + r at step (s, r), so one
// ds_read_b128 per operand tile feeds four MFMA steps.
//
// D has the vector index on the lane (j) axis.  That is what lets the
// epilogues work per lane: a lane holds 16 coordinates of ONE vector per tile,
// builds its share of the packed words locally and merges with the other
// half-wave through one cross-lane exchange.
//
// Pieces (NP > 0).  The same contraction can run on the bf16 matrix cores: both fp32 operands are split
// into NP exact bf16 pieces while they are staged into LDS (a bf16 input is one piece as it stands) and the
// piece products of combined weight >= 2^(-8 (NP - 1)) are summed in the fp32 accumulator with
// v_mfma_f32_32x32x16_bf16, whose D layout is the one above, so the epilogues do not change.  NP = 3
// keeps W exact (three pieces) against the two leading pieces of an fp32 vector or the one of a bf16 vector
// (five resp. three products: y to 8e-6 |x| at worst, see mfma_tile); NP = 2 (three products) is used where
// only signs are kept.
#include "tq_bf3.h"

#include <cstdlib>
#include <type_traits>

namespace tq {


constexpr int TM = 128;      // rows of W per workgroup
constexpr int TN = 128;      // vectors per workgroup
constexpr int BK = 32;       // k per LDS stage
constexpr int LDS_LD = 36;   // padded row stride (floats)
constexpr int P_LD = 104;    // pieces: bf16 per staged row, [piece][32 k] + 8 padding (208 bytes: conflict-free 16-byte reads)
constexpr int XCDS = 8;

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// IMG (pieces only): W1 comes from its image (GemmArgs::W1_image) instead of being split in every workgroup
template <int NKIND, int EKIND, int BITS, int NP, bool IMG>
__global__ __launch_bounds__(256, 2) void gemm_kernel(const GemmArgs a, const int tiles_m,
                                                   const int tiles_n, const int per_xcd) {
  // two staging buffers of [TM + TN][LDS_LD] floats: one is read by the MFMAs while the next
  // k-tile is written into the other, so a k-step costs a single workgroup barrier
  extern __shared__ __attribute__((aligned(16))) float stage_s[];
  __shared__ float row_ss[TN];
  __shared__ float cent_s[16];
  __shared__ float thr_s[16];

  // workgroup -> tile.  Consecutive workgroup ids go round-robin over the 8
  // XCDs; give every XCD a contiguous range of tiles, m fastest, so the m
  // tiles that re-read the same block of vectors share one L2.
  const int total = tiles_m * tiles_n;
  const int logical = (int)(blockIdx.x % XCDS) * per_xcd + (int)(blockIdx.x / XCDS);
  if (logical >= total) return;
  const int tile_m = logical % tiles_m;
  const int tile_n = logical / tiles_m;
  const int group = blockIdx.y;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, h = lane >> 5;

  const int m0 = tile_m * TM;
  const int64_t n0 = (int64_t)tile_n * TN;
  const int64_t vec_base = (int64_t)group * a.n;  // first vector row of this group

  const int kt_per_seg = a.d / BK;
  const int n_kt = kt_per_seg * a.segs;
  const int words_per_row = kt_per_seg * BITS;

  // staging: thread (row = tid/8 + 32p, col4 = tid%8) moves one 16-byte piece
  const int srow = tid >> 3;
  const int scol = (tid & 7) * 4;

  // the codebook goes to LDS once; indexing the argument block by thread id reads it from
  // memory, so its 31 entries never occupy scalar registers
  if ((NKIND == N_CODE || EKIND == E_QUANT) && tid < 16) {
    cent_s[tid] = a.cb.c[tid];
    thr_s[tid] = tid < 15 ? a.cb.t[tid] : 0.f;
  }

  // Addresses are a per-tile uniform base plus a small per-thread offset.  Rows past the end
  // of either operand are clamped onto the last valid row: what they produce is never stored.
  const int rows_m = min(TM, a.M - m0);
  const int rows_n = (int)min((int64_t)TN, a.n - n0);
  const float* const W1 = a.W1 + (int64_t)group * a.w_group_stride + (int64_t)m0 * a.ldw;
  const float* const W2 =
      (a.segs > 1) ? a.W2 + (int64_t)group * a.w_group_stride + (int64_t)m0 * a.ldw : nullptr;
  const float* const Xf = reinterpret_cast<const float*>(a.X) + (NKIND == N_F32 ? (vec_base + n0) * a.ldx : 0);
  const uint16_t* const Xh =
      reinterpret_cast<const uint16_t*>(a.X) + (NKIND == N_BF16 ? (vec_base + n0) * a.ldx : 0);
  const uint32_t* const Ci = a.idx + (NKIND == N_CODE ? (vec_base + n0) * words_per_row : 0);
  const uint32_t* const Cq = a.qjl + ((NKIND == N_CODE && a.segs > 1) ? (vec_base + n0) * kt_per_seg : 0);
  uint32_t woff[4], noff[4], qoff[4];
  float kg[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const uint32_t rm = (uint32_t)min(srow + 32 * p, rows_m - 1);
    const uint32_t rn = (uint32_t)min(srow + 32 * p, rows_n - 1);
    woff[p] = rm * (uint32_t)a.ldw + scol;
    noff[p] = (NKIND == N_CODE) ? rn * (uint32_t)words_per_row : rn * (uint32_t)a.ldx + scol;
    qoff[p] = rn * (uint32_t)kt_per_seg;
    if (NKIND == N_CODE && a.segs > 1) kg[p] = a.kappa * a.gamma[vec_base + n0 + rn];
  }

  f32x4 wreg[4];  // native vectors: these stay in registers
  uint32_t nreg[16];
  // W from its image (pieces only): a row's k-tile is NP * 64 contiguous bytes, [piece][32 k]; chunk c = i * 256 + tid
  // of the tile's 128 * NP * 4 chunks of 16 bytes is (row c / (4 NP), piece, eight k)
  constexpr int NCH = IMG ? 2 * NP : 1;
  constexpr bool w_image = IMG;
  const u32x4* const Wimg = reinterpret_cast<const u32x4*>(a.W1_image);
  uint32_t ioff[NCH], loff[NCH];
  u32x4 wimg[NCH];
  if constexpr (IMG) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = i * 256 + tid, row = c / (4 * NP), within = c % (4 * NP);
      const uint32_t rm = (uint32_t)min(row, rows_m - 1);
      ioff[i] = ((uint32_t)(m0 + rm) * (uint32_t)kt_per_seg) * (4 * NP) + within;  // in chunks; + kt * 4 NP per k-tile
      loff[i] = row * P_LD + (within >> 2) * 32 + (within & 3) * 8;               // in bf16 elements
    }
  }
  float ss[4] = {0.f, 0.f, 0.f, 0.f};

  // global -> registers for k-tile kt; SEG (0: rotated codebook part, 1: sign sketch part)
  // only matters for packed codes and is a compile-time constant of each loop below
  auto load_tiles = [&](auto seg_c, int kt) {
    constexpr int SEG = decltype(seg_c)::value;
    const int g = kt - SEG * kt_per_seg;
    const float* W = (SEG ? W2 : W1) + g * BK;
    if constexpr (IMG) {
#pragma unroll
      for (int i = 0; i < NCH; ++i) wimg[i] = Wimg[ioff[i] + (uint32_t)g * (4 * NP)];
    } else {
#pragma unroll
      for (int p = 0; p < 4; ++p) wreg[p] = *reinterpret_cast<const f32x4*>(W + woff[p]);
    }
    if (NKIND == N_F32) {
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const uint4 v = *reinterpret_cast<const uint4*>(Xf + g * BK + noff[p]);
        nreg[4 * p + 0] = v.x; nreg[4 * p + 1] = v.y; nreg[4 * p + 2] = v.z; nreg[4 * p + 3] = v.w;
      }
    } else if (NKIND == N_BF16) {
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const uint2 v = *reinterpret_cast<const uint2*>(Xh + g * BK + noff[p]);
        nreg[4 * p + 0] = v.x; nreg[4 * p + 1] = v.y;
      }
    } else if (SEG == 0) {
      const uint32_t* C = Ci + g * BITS;
#pragma unroll
      for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int pl = 0; pl < BITS; ++pl) nreg[4 * p + pl] = C[noff[p] + pl];
    } else {
      const uint32_t* C = Cq + g;
#pragma unroll
      for (int p = 0; p < 4; ++p) nreg[4 * p] = C[qoff[p]];
    }
  };

  // registers -> staging buffer (decoding packed codes on the way)
  auto store_tiles = [&](auto seg_c, float* Ws, float* Ns) {
    constexpr int SEG = decltype(seg_c)::value;
    if constexpr (NP > 0) {
      // both tiles as bf16 pieces, [row][piece][k]
      unsigned short* const Wp = reinterpret_cast<unsigned short*>(Ws);
      unsigned short* const Xp = reinterpret_cast<unsigned short*>(Ns);
      if constexpr (IMG) {
#pragma unroll
        for (int i = 0; i < NCH; ++i) *reinterpret_cast<u32x4*>(Wp + loff[i]) = wimg[i];
      }
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        uint32_t lo[3], hi[3];
        if constexpr (!IMG) {
          split3_pair(f32x2{wreg[p][0], wreg[p][1]}, lo[0], lo[1], lo[2]);
          split3_pair(f32x2{wreg[p][2], wreg[p][3]}, hi[0], hi[1], hi[2]);
#pragma unroll
          for (int pc = 0; pc < NP; ++pc)
            *reinterpret_cast<uint2*>(Wp + (srow + 32 * p) * P_LD + pc * 32 + scol) = make_uint2(lo[pc], hi[pc]);
        }
        if (NKIND == N_BF16) {
          const float x0 = bf16_lo(nreg[4 * p]), x1 = bf16_hi(nreg[4 * p]), x2 = bf16_lo(nreg[4 * p + 1]), x3 = bf16_hi(nreg[4 * p + 1]);
          ss[p] += x0 * x0 + x1 * x1 + x2 * x2 + x3 * x3;
          *reinterpret_cast<uint2*>(Xp + (srow + 32 * p) * P_LD + scol) = make_uint2(nreg[4 * p], nreg[4 * p + 1]);
        } else {
          const float x0 = __uint_as_float(nreg[4 * p]), x1 = __uint_as_float(nreg[4 * p + 1]);
          const float x2 = __uint_as_float(nreg[4 * p + 2]), x3 = __uint_as_float(nreg[4 * p + 3]);
          ss[p] += x0 * x0 + x1 * x1 + x2 * x2 + x3 * x3;
          // the streamed vector as its two leading pieces (see mfma_tile)
          split2_pair(f32x2{x0, x1}, lo[0], lo[1]);
          split2_pair(f32x2{x2, x3}, hi[0], hi[1]);
#pragma unroll
          for (int pc = 0; pc < 2; ++pc)
            *reinterpret_cast<uint2*>(Xp + (srow + 32 * p) * P_LD + pc * 32 + scol) = make_uint2(lo[pc], hi[pc]);
        }
      }
      return;
    }
#pragma unroll
    for (int p = 0; p < 4; ++p)
      *reinterpret_cast<f32x4*>(&Ws[(srow + 32 * p) * LDS_LD + scol]) = wreg[p];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      float4 v;
      if (NKIND == N_F32) {
        v = make_float4(__uint_as_float(nreg[4 * p]), __uint_as_float(nreg[4 * p + 1]),
                        __uint_as_float(nreg[4 * p + 2]), __uint_as_float(nreg[4 * p + 3]));
      } else if (NKIND == N_BF16) {
        v = make_float4(bf16_lo(nreg[4 * p]), bf16_hi(nreg[4 * p]), bf16_lo(nreg[4 * p + 1]),
                        bf16_hi(nreg[4 * p + 1]));
      } else {
        float e[4];
        if (SEG == 0) {
          // four coordinates at once: each plane's 4 bits are spread to one bit per byte by a
          // multiply (bit i lands at 8i), planes are merged so that byte q holds 4*code_q,
          // which is the byte offset into the LDS centroid table
          uint32_t x = 0;
#pragma unroll
          for (int pl = 0; pl < BITS; ++pl) {
            const uint32_t nibble = (nreg[4 * p + pl] >> scol) & 0xFu;
            x |= ((nibble * 0x00204081u) & 0x01010101u) << (pl + 2);
          }
#pragma unroll
          for (int q = 0; q < 4; ++q)
            e[q] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(cent_s) + ((x >> (8 * q)) & 0xFFu));
        } else {
          // +-kappa*gamma: the sign bit comes from the inverted qjl bit
          const uint32_t zn = ~nreg[4 * p] >> scol;
#pragma unroll
          for (int q = 0; q < 4; ++q)
            e[q] = __uint_as_float(((zn << (31 - q)) & 0x80000000u) | __float_as_uint(kg[p]));
        }
        v = make_float4(e[0], e[1], e[2], e[3]);
      }
      if (NKIND != N_CODE) ss[p] += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
      *reinterpret_cast<float4*>(&Ns[(srow + 32 * p) * LDS_LD + scol]) = v;
    }
  };

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  constexpr int BUF = NP > 0 ? (TM + TN) * P_LD / 2 : (TM + TN) * LDS_LD;  // floats per staging buffer
  constexpr int W_PART = NP > 0 ? TM * P_LD / 2 : TM * LDS_LD;           // floats of its W tile
  auto mfma_tile = [&](const float* Ws, const float* Ns) {
    if constexpr (NP > 0) {
      const unsigned short* const Wp = reinterpret_cast<const unsigned short*>(Ws);
      const unsigned short* const Xp = reinterpret_cast<const unsigned short*>(Ns);
      // Pieces of the streamed operand: a bf16 vector is one; an fp32 vector is taken as its two leading pieces,
      // x = x1 + x2 + dx with |dx_k| <= 2^-17 |x_k| (2^-18.6 in the root mean square).  What that leaves out of
      // y = W x is W dx: at most 2^-17 |W_j| |x| in any one coordinate (7.6e-6 for a unit vector against a row of a
      // rotation, inside the 1e-5 within which a bucket decision may differ from the exact one), and, W being
      // orthogonal there, 2^-17 |x| in norm over all coordinates together, so for no input more than a few in 10^5
      // decisions can sit that close to a cell boundary.  W itself keeps all NP pieces.
      constexpr int NPX = NKIND == N_BF16 ? 1 : 2;
#pragma unroll
      for (int s = 0; s < 2; ++s) {  // 16 values of k per step: lane half h holds k = 16 s + 8 h + 0..7
        bf16x8 av[2][NP], bv[2][NPX];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
          for (int pc = 0; pc < NP; ++pc)
            av[t][pc] = *reinterpret_cast<const bf16x8*>(Wp + (wm * 64 + t * 32 + l32) * P_LD + pc * 32 + 16 * s + 8 * h);
#pragma unroll
          for (int pc = 0; pc < NPX; ++pc)
            bv[t][pc] = *reinterpret_cast<const bf16x8*>(Xp + (wn * 64 + t * 32 + l32) * P_LD + pc * 32 + 16 * s + 8 * h);
        }
        // products of pieces pa, pb with pa + pb < NP, smallest first; the four accumulators in turn
#pragma unroll
        for (int w = NP - 1; w >= 0; --w)
#pragma unroll
          for (int pb = 0; pb < NPX; ++pb) {
            const int pa = w - pb;
            if (pa < 0) continue;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
              for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i][pa], bv[j][pb], acc[i][j], 0, 0, 0);
          }
      }
      return;
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      float4 av[2], bv[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        av[t] = *reinterpret_cast<const float4*>(&Ws[(wm * 64 + t * 32 + l32) * LDS_LD + 8 * s + 4 * h]);
        bv[t] = *reinterpret_cast<const float4*>(&Ns[(wn * 64 + t * 32 + l32) * LDS_LD + 8 * s + 4 * h]);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i].x, bv[j].x, acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i].y, bv[j].y, acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i].z, bv[j].z, acc[i][j], 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i].w, bv[j].w, acc[i][j], 0, 0, 0);
        }
    }
  };

  // Step kt: the registers hold k-tile kt+1 (segment SN); it goes into the buffer that step
  // kt-1 read, k-tile kt+2 (segment SF) is requested, and the MFMAs run on k-tile kt.  The
  // barrier that ends the step both publishes the new buffer and retires the old one.
  auto steps = [&](int kt_begin, int kt_end, auto sn_c, auto sf_c) {
    if constexpr (NP > 0) {
      // pieces: ONE staging buffer (two would leave room for a single workgroup per compute unit, and the second
      // workgroup hides more than the second buffer does): MFMAs, barrier, refill, barrier
      for (int kt = kt_begin; kt < kt_end; ++kt) {
        mfma_tile(stage_s, stage_s + W_PART);
        __syncthreads();
        if (kt + 1 < n_kt) store_tiles(sn_c, stage_s, stage_s + W_PART);
        if (kt + 2 < n_kt) load_tiles(sf_c, kt + 2);
        __syncthreads();
      }
      return;
    }
    for (int kt = kt_begin; kt < kt_end; ++kt) {
      float* const cur = stage_s + (kt & 1) * BUF;
      float* const nxt = stage_s + ((kt + 1) & 1) * BUF;
      if (kt + 1 < n_kt) store_tiles(sn_c, nxt, nxt + W_PART);
      if (kt + 2 < n_kt) load_tiles(sf_c, kt + 2);
      mfma_tile(cur, cur + W_PART);
      __syncthreads();
    }
  };
  using S0 = std::integral_constant<int, 0>;
  using S1 = std::integral_constant<int, 1>;

  load_tiles(S0{}, 0);
  __syncthreads();  // cent_s visible before the first decode
  store_tiles(S0{}, stage_s, stage_s + W_PART);
  if (NKIND == N_CODE && a.segs > 1) {
    if (n_kt > 1) {
      if (kt_per_seg > 1) load_tiles(S0{}, 1);
      else load_tiles(S1{}, 1);
    }
    __syncthreads();
    steps(0, kt_per_seg - 2, S0{}, S0{});
    if (kt_per_seg >= 2) steps(kt_per_seg - 2, kt_per_seg - 1, S0{}, S1{});
    steps(kt_per_seg - 1, n_kt, S1{}, S1{});
  } else {
    if (n_kt > 1) load_tiles(S0{}, 1);
    __syncthreads();
    steps(0, n_kt, S0{}, S0{});
  }

  // squared norms of the streamed rows: 8 neighbouring lanes share a row
  if (NKIND != N_CODE) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      float v = ss[p];
      v += __shfl_xor(v, 1);
      v += __shfl_xor(v, 2);
      v += __shfl_xor(v, 4);
      if ((tid & 7) == 0) row_ss[srow + 32 * p] = v;
    }
    __syncthreads();
    if (a.rownorm_out != nullptr && tile_m == 0 && tid < TN) {
      const int64_t i = n0 + tid;
      if (i < a.n) a.rownorm_out[vec_base + i] = sqrtf(row_ss[tid]);
    }
  }

  // ------------------------------- epilogue -------------------------------
  // The epilogue takes the codebook from LDS into vector registers: with up to 31 table
  // entries, the argument block and the compare masks all live at once the scalar file would
  // overflow (spills through v_writelane), while vector registers are plentiful here.
  constexpr int NT = (EKIND == E_QUANT) ? (1 << BITS) - 1 : 0;
  float tv[NT > 0 ? NT : 1], cv[NT + 1];
  if (EKIND == E_QUANT) {
#pragma unroll
    for (int j = 0; j < NT; ++j) tv[j] = thr_s[j];
#pragma unroll
    for (int j = 0; j <= NT; ++j) cv[j] = cent_s[j];
  }
  if (EKIND == E_STORE_T) {
    // D is held with the vector on the lane axis, so a lane owns 4 consecutive m of one
    // vector: stored directly that is 16 bytes per lane at a row stride.  Instead the tile is
    // turned in LDS, 64 vectors at a time (the two wavefronts with the same wn), and written
    // out by all threads along m.
    constexpr int T_LD = TM + 4;
    float* const T = stage_s;  // [64][T_LD] <= (TM + TN) * LDS_LD floats
#pragma unroll 1
    for (int w = 0; w < 2; ++w) {
      __syncthreads();
      if (wn == w) {
#pragma unroll
        for (int tn = 0; tn < 2; ++tn) {
          const int64_t i = n0 + wn * 64 + tn * 32 + l32;
          float scale = 1.f;
          if (a.scale_in != nullptr && i < a.n) scale = a.scale_in[vec_base + i];
#pragma unroll
          for (int tm = 0; tm < 2; ++tm)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              const floatx16& c = acc[tm][tn];
              *reinterpret_cast<float4*>(&T[(tn * 32 + l32) * T_LD + wm * 64 + tm * 32 + 8 * k + 4 * h]) =
                  make_float4(c[4 * k] * scale, c[4 * k + 1] * scale, c[4 * k + 2] * scale, c[4 * k + 3] * scale);
            }
        }
      }
      __syncthreads();
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int f = tid + 256 * j;  // 64 rows x 32 float4
        const int row = f >> 5, c4 = f & 31;
        const int64_t i = n0 + w * 64 + row;
        const int m = m0 + 4 * c4;
        if (i < a.n && m < a.M)
          *reinterpret_cast<float4*>(a.out + (vec_base + i) * a.ldo + m) =
              *reinterpret_cast<const float4*>(&T[row * T_LD + 4 * c4]);
      }
    }
    return;
  }

#pragma unroll
  for (int tn = 0; tn < 2; ++tn) {
    const int vloc = wn * 64 + tn * 32 + l32;
    const int64_t i = n0 + vloc;
    const bool valid = i < a.n;
    float scale = 1.f;
    if (EKIND == E_QUANT) {
      if (a.normalise) {
        const float nu = sqrtf(row_ss[vloc]);
        scale = nu > 0.f ? 1.f / nu : 0.f;
      }
    } else if (EKIND == E_STORE_T || EKIND == E_STORE_N) {
      if (a.scale_in != nullptr && valid) scale = a.scale_in[vec_base + i];
    }
#pragma unroll
    for (int tm = 0; tm < 2; ++tm) {
      __builtin_amdgcn_sched_barrier(0);  // one tile's epilogue at a time (register pressure)
      const int mb = m0 + wm * 64 + tm * 32;  // first row of this 32x32 tile
      const floatx16& c = acc[tm][tn];
      if (EKIND == E_STORE_T) {
        // handled below, through LDS, so that rows leave the chip as whole 512-byte lines
      } else if (EKIND == E_STORE_N) {
        if (valid) {
          float* o = a.out + (int64_t)group * a.out_group_stride + i;
#pragma unroll
          for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int m = mb + 8 * k + 4 * h + r;
              if (m < a.M) o[(int64_t)m * a.ldo] = c[4 * k + r] * scale;
            }
        }
      } else {
        constexpr int PL = (EKIND == E_SIGN) ? 1 : BITS;
        constexpr int PLN = PL > 0 ? PL : 1;
        // a 4-bit nibble of each bit plane per k, most significant element first; bit p of the
        // bucket number is the XOR of the compare masks at positions j = 2^p - 1 (mod 2^p)
        uint32_t nib[4][PLN];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          float e[4];
#pragma unroll
          for (int pl = 0; pl < PLN; ++pl) nib[k][pl] = 0u;
#pragma unroll
          for (int r = 3; r >= 0; --r) {
            bool bit[PLN];
#pragma unroll
            for (int pl = 0; pl < PLN; ++pl) bit[pl] = false;
            if (EKIND == E_SIGN) {
              bit[0] = c[4 * k + r] >= 0.f;
              e[r] = 0.f;
            } else {
              const float y = c[4 * k + r] * scale;
              float yt = cv[0];
#pragma unroll
              for (int j = 0; j < NT; ++j) {
                const bool ge = y >= tv[j];
                yt = ge ? cv[j + 1] : yt;
#pragma unroll
                for (int pl = 0; pl < PL; ++pl)
                  if ((j & ((1 << pl) - 1)) == (1 << pl) - 1) bit[pl] = bit[pl] != ge;
              }
              float ev = y - yt;
              asm volatile("" : "+v"(ev));  // computed here, while the compare masks are live
              e[r] = ev;
            }
#pragma unroll
            for (int pl = 0; pl < PL; ++pl) {
              nib[k][pl] = nib[k][pl] + nib[k][pl] + (bit[pl] ? 1u : 0u);
              asm volatile("" : "+v"(nib[k][pl]));  // consume this element's masks now (scalar registers)
            }
          }
          if (EKIND == E_QUANT && a.resid_out != nullptr) {
            const int m = mb + 8 * k + 4 * h;
            if (valid && m < a.M)
              *reinterpret_cast<float4*>(a.resid_out + (vec_base + i) * (int64_t)a.d + m) =
                  make_float4(e[0], e[1], e[2], e[3]);
          }
        }
        uint32_t piece[PLN];
#pragma unroll
        for (int pl = 0; pl < PLN; ++pl)
          piece[pl] = nib[0][pl] | (nib[1][pl] << 8) | (nib[2][pl] << 16) | (nib[3][pl] << 24);
        // merge the two half-waves (rows 8k+r and 8k+4+r) and let half tm&1 store
#pragma unroll
        for (int pl = 0; pl < PL; ++pl) {
          uint32_t w = piece[pl] << (4 * h);
          w |= (uint32_t)__shfl_xor((int)w, 32);
          const int g = mb >> 5;
          if (valid && mb < a.M && h == (tm & 1))
            a.words_out[(vec_base + i) * (int64_t)(kt_per_seg * PL) + g * PL + pl] = w;
        }
      }
    }
  }
}

// W (M rows of d fp32 values, row stride ldw) as its np leading bf16 pieces in the order the piece kernels copy
// it: [row][k / 32][piece][32 k].  Thread = four consecutive k of one row.
template <int NP>
__global__ __launch_bounds__(256) void gemm_image_kernel(const float* W, int64_t ldw, int M, int d, unsigned short* out) {
  const int64_t e = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (e >= (int64_t)M * d) return;
  const int64_t row = e / d;
  const int k = (int)(e % d);
  const f32x4 v = *reinterpret_cast<const f32x4*>(W + row * ldw + k);
  uint32_t lo[3], hi[3];
  split3_pair(f32x2{v[0], v[1]}, lo[0], lo[1], lo[2]);
  split3_pair(f32x2{v[2], v[3]}, hi[0], hi[1], hi[2]);
  unsigned short* const dst = out + (row * (d / BK) + k / BK) * (NP * BK) + (k % BK);
#pragma unroll
  for (int pc = 0; pc < NP; ++pc) *reinterpret_cast<uint2*>(dst + pc * BK) = make_uint2(lo[pc], hi[pc]);
}

template <int NKIND, int EKIND, int BITS, int NP = 0, bool IMG = false>
static hipError_t launch_one(const GemmArgs& a, int n_groups, hipStream_t stream) {
  const int tiles_m = (a.M + TM - 1) / TM;
  const int64_t tiles_n64 = (a.n + TN - 1) / TN;
  if (tiles_n64 * tiles_m > (int64_t)1 << 30) return hipErrorInvalidValue;
  const int tiles_n = (int)tiles_n64;
  const int total = tiles_m * tiles_n;
  if (total == 0 || n_groups == 0) return hipSuccess;
  const int per_xcd = (total + XCDS - 1) / XCDS;
  dim3 grid(per_xcd * XCDS, n_groups, 1);
  constexpr int lds_bytes = NP > 0 ? (TM + TN) * P_LD * 2 : 2 * (TM + TN) * LDS_LD * (int)sizeof(float);  // above the 64 KB default limit
  static LdsLimit lds_limit;  // per instantiation: the limit is raised once per device
  if (const hipError_t e = raise_lds_limit(lds_limit, reinterpret_cast<const void*>(&gemm_kernel<NKIND, EKIND, BITS, NP, IMG>), lds_bytes); e != hipSuccess) return e;
  hipLaunchKernelGGL((gemm_kernel<NKIND, EKIND, BITS, NP, IMG>), grid, dim3(256), lds_bytes, stream, a, tiles_m,
                     tiles_n, per_xcd);
  return hipGetLastError();
}

template <int NKIND, int EKIND, int NP = 0, bool IMG = false>
static hipError_t launch_bits(int bits, const GemmArgs& a, int g, hipStream_t s) {
  switch (bits) {
    case 0: return launch_one<NKIND, EKIND, 0, NP, IMG>(a, g, s);
    case 1: return launch_one<NKIND, EKIND, 1, NP, IMG>(a, g, s);
    case 2: return launch_one<NKIND, EKIND, 2, NP, IMG>(a, g, s);
    case 3: return launch_one<NKIND, EKIND, 3, NP, IMG>(a, g, s);
    case 4: return launch_one<NKIND, EKIND, 4, NP, IMG>(a, g, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_gemm(NKind nk, EKind ek, int bits, const GemmArgs& a, int n_groups,
                       hipStream_t stream) {
  // only the combinations the library uses are instantiated
  // the quantiser's two contractions on the bf16 matrix cores when the caller asks for pieces: the rotation with
  // three pieces (fp32 accuracy), the sketch (signs only) with two
  const bool pieces = a.pieces != 0;
  const bool img = pieces && a.W1_image != nullptr && n_groups == 1 && (reinterpret_cast<uintptr_t>(a.W1_image) & 15u) == 0;
  if (img && nk == N_F32 && ek == E_QUANT) return launch_bits<N_F32, E_QUANT, 3, true>(bits, a, n_groups, stream);
  if (img && nk == N_BF16 && ek == E_QUANT) return launch_bits<N_BF16, E_QUANT, 3, true>(bits, a, n_groups, stream);
  if (img && nk == N_F32 && ek == E_SIGN) return launch_one<N_F32, E_SIGN, 0, 2, true>(a, n_groups, stream);
  if (pieces && nk == N_F32 && ek == E_QUANT) return launch_bits<N_F32, E_QUANT, 3>(bits, a, n_groups, stream);
  if (pieces && nk == N_BF16 && ek == E_QUANT) return launch_bits<N_BF16, E_QUANT, 3>(bits, a, n_groups, stream);
  if (pieces && nk == N_F32 && ek == E_SIGN) return launch_one<N_F32, E_SIGN, 0, 2>(a, n_groups, stream);
  if (nk == N_F32 && ek == E_QUANT) return launch_bits<N_F32, E_QUANT>(bits, a, n_groups, stream);
  if (nk == N_BF16 && ek == E_QUANT) return launch_bits<N_BF16, E_QUANT>(bits, a, n_groups, stream);
  if (nk == N_F32 && ek == E_SIGN) return launch_one<N_F32, E_SIGN, 0>(a, n_groups, stream);
  if (nk == N_F32 && ek == E_STORE_T) return launch_one<N_F32, E_STORE_T, 0>(a, n_groups, stream);
  if (nk == N_CODE && ek == E_STORE_T) return launch_bits<N_CODE, E_STORE_T>(bits, a, n_groups, stream);
  if (nk == N_CODE && ek == E_STORE_N) return launch_bits<N_CODE, E_STORE_N>(bits, a, n_groups, stream);
  return hipErrorInvalidValue;
}

size_t gemm_image_bytes(int M, int d, int np) { return (size_t)M * d * np * 2; }

hipError_t launch_gemm_image(const float* W, int64_t ldw, int M, int d, int np, void* image, hipStream_t stream) {
  if (M <= 0 || d <= 0 || d % BK != 0 || ldw % 4 != 0 || (np != 2 && np != 3)) return hipErrorInvalidValue;
  const int64_t threads = (int64_t)M * d / 4;
  const dim3 grid((unsigned)((threads + 255) / 256));
  if (np == 3) hipLaunchKernelGGL(gemm_image_kernel<3>, grid, dim3(256), 0, stream, W, ldw, M, d, static_cast<unsigned short*>(image));
  else hipLaunchKernelGGL(gemm_image_kernel<2>, grid, dim3(256), 0, stream, W, ldw, M, d, static_cast<unsigned short*>(image));
  return hipGetLastError();
}

}  // namespace tq
