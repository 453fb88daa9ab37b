// Quantisation at d = 128 for a small number of vectors: the tokens a decoding
// step appends to a key cache (Sec. 4.3), or any batch too small to fill the
// chip with the streaming kernel of tq_d128.hip.
//
// There, one wavefront carries a block of 32 vectors through both contractions
// (512 MFMAs in a row, 14 us) behind a 128 KB parameter load into LDS: fine when
// every wavefront of the chip has blocks to chew on, a long latency chain when
// there are only a few blocks.  Here a whole workgroup of 8 wavefronts shares
// ONE block: wavefront w computes output tile w % 4 (32 coordinates) over half
// w / 4 of the contraction index, reading its slice of Pi / S Pi^T straight
// from L2 into registers (requested for both contractions before anything
// else), and the two halves are added through LDS.  The residual goes through
// LDS once, because the second contraction needs all 128 coordinates of it.
// Per wavefront that is 2 x 32 MFMAs and three workgroup barriers.
//
// Operand layout as in tq_gemm.hip / tq_d128.hip: vector on the MFMA lane axis,
// lane half h owns k in [64 h, 64 h + 64) of which this wavefront takes
// [64 h + 32 kh, 64 h + 32 kh + 32); accumulator register 4 k + r of tile t is
// coordinate 32 t + 8 k + 4 h + r of vector lane % 32.
#include "tq_d128_tile.h"

namespace tq {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct QuantSmallArgs {
  const void* X;
  int64_t ldx;
  int64_t n;
  const float* Pi;
  const float* SPiT;
  uint32_t* idx;
  uint32_t* qjl;
  float* gamma;
  float* norm;
  int64_t out_first, out_step;  // vector i is written as code row out_first + i * out_step
  int normalise;
  int gs_hi;  // two instances (MIXED): coordinate groups [0, gs_hi) belong to instance hi
  Codebook cb;
  Codebook cb_hi;
};

constexpr int E_LD = 132;  // padded row stride of the residual tile in LDS

// MIXED: two instances over a split of the rotated coordinates (Sec. 4.3): tiles [0, gs_hi)
// are quantised with BITS + 1 bits and the codebook cb_hi, the others with BITS and cb; each
// instance normalises by the norm of its own rotated coordinates (equal to that of its own
// channels, the blocks of Pi being orthogonal) and keeps its own residual norm.
template <int BITS, bool PROD, bool BF16IN, bool MIXED>
__global__ __launch_bounds__(512) void quant128_small_kernel(const QuantSmallArgs a) {
  __shared__ __attribute__((aligned(16))) float part1_s[4 * 16 * 64];  // upper-half partial tiles [tile][register][lane]
  __shared__ __attribute__((aligned(16))) float part2_s[PROD ? 4 * 16 * 64 : 64];
  __shared__ __attribute__((aligned(16))) float e_s[PROD ? 32 * E_LD : 4];  // residual [vector][coordinate]
  __shared__ float ss_s[4][32];  // partial sums of squares: of x by k-half, or (MIXED) of y by tile
  __shared__ float g2_s[4][32];  // partial squared residual norms by tile
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, h = lane >> 5;
  const int mt = wave & 3, kh = wave >> 2;
  const int k0 = 64 * h + 32 * kh;  // first contraction index of this lane
  const int gs = MIXED ? a.gs_hi : 0;
  const bool hi = MIXED && mt < gs;  // uniform
  const int wpr = MIXED ? gs * (BITS + 1) + (4 - gs) * BITS : 4 * BITS;
  const int woff = MIXED ? (mt < gs ? mt * (BITS + 1) : gs * (BITS + 1) + (mt - gs) * BITS) : mt * BITS;

  // ---- this wavefront's slices of both parameter matrices, requested up front and kept ----
  f32x4 pa[8], sa[8];
  {
    const float* prow = a.Pi + (32 * mt + l32) * 128 + k0;
#pragma unroll
    for (int j = 0; j < 8; ++j) pa[j] = *reinterpret_cast<const f32x4*>(prow + 4 * j);
  }
  constexpr int RAW = BF16IN ? 4 : 8;  // 16-byte loads per lane for its quarter row
  u32x4 raw[RAW];
  const int64_t n_blocks = (a.n + 31) / 32;
  auto load_raw = [&](int64_t blk) {
    const int64_t i = blk * 32 + l32;
    const char* src = reinterpret_cast<const char*>(a.X) + ((i < a.n ? i : a.n - 1) * a.ldx + k0) * (BF16IN ? 2 : 4);
#pragma unroll
    for (int v = 0; v < RAW; ++v) raw[v] = *reinterpret_cast<const u32x4*>(src + 16 * v);
  };
  load_raw(blockIdx.x);
  if (PROD) {
    const float* srow = a.SPiT + (32 * mt + l32) * 128 + k0;
#pragma unroll
    for (int j = 0; j < 8; ++j) sa[j] = *reinterpret_cast<const f32x4*>(srow + 4 * j);
  }

  for (int64_t blk = blockIdx.x; blk < n_blocks; blk += gridDim.x) {
    const int64_t i = blk * 32 + l32;
    const bool valid = i < a.n;
    const int64_t oi = a.out_first + i * a.out_step;  // code row
    float xb[32];
    if (BF16IN) {
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        xb[8 * v + 0] = __uint_as_float(raw[v].x << 16); xb[8 * v + 1] = __uint_as_float(raw[v].x & 0xffff0000u);
        xb[8 * v + 2] = __uint_as_float(raw[v].y << 16); xb[8 * v + 3] = __uint_as_float(raw[v].y & 0xffff0000u);
        xb[8 * v + 4] = __uint_as_float(raw[v].z << 16); xb[8 * v + 5] = __uint_as_float(raw[v].z & 0xffff0000u);
        xb[8 * v + 6] = __uint_as_float(raw[v].w << 16); xb[8 * v + 7] = __uint_as_float(raw[v].w & 0xffff0000u);
      }
    } else {
#pragma unroll
      for (int v = 0; v < 8; ++v) {
        xb[4 * v] = __uint_as_float(raw[v].x); xb[4 * v + 1] = __uint_as_float(raw[v].y);
        xb[4 * v + 2] = __uint_as_float(raw[v].z); xb[4 * v + 3] = __uint_as_float(raw[v].w);
      }
    }
    // the next block's rows travel while this one is worked on
    if (blk + gridDim.x < n_blocks) load_raw(blk + gridDim.x);

    // ---- norm of x: tile-0 wavefronts add up their quarter of each row --------------------
    if (!MIXED && a.normalise && mt == 0) {
      float s0 = 0.f, s1 = 0.f;
#pragma unroll
      for (int k = 0; k < 32; k += 2) {
        s0 = fmaf(xb[k], xb[k], s0);
        s1 = fmaf(xb[k + 1], xb[k + 1], s1);
      }
      float ss = s0 + s1;
      ss += __shfl_xor(ss, 32);
      if (h == 0) ss_s[kh][l32] = ss;
    }

    // ---- Y = Pi X: this wavefront's tile over its half of k --------------------------------
    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[j].x, xb[4 * j + 0], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[j].y, xb[4 * j + 1], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[j].z, xb[4 * j + 2], acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[j].w, xb[4 * j + 3], acc, 0, 0, 0);
    }
    if (kh == 1) {
#pragma unroll
      for (int r = 0; r < 16; ++r) part1_s[(mt * 16 + r) * 64 + lane] = acc[r];
    }
    __syncthreads();

    if (MIXED) {
      // the norms of the two instances come from the rotated coordinates: per-tile sums first
      if (kh == 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] += part1_s[(mt * 16 + r) * 64 + lane];
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          s0 = fmaf(acc[r], acc[r], s0);
          s1 = fmaf(acc[r + 1], acc[r + 1], s1);
        }
        float ss = s0 + s1;
        ss += __shfl_xor(ss, 32);
        if (h == 0) ss_s[mt][l32] = ss;
      }
      __syncthreads();
    }

    if (kh == 0) {
      float nu = 1.f, nu_other = 1.f, inv = 1.f;
      if (MIXED) {
        float s_hi = 0.f, s_lo = 0.f;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const float v = ss_s[t][l32];
          s_hi += t < gs ? v : 0.f;
          s_lo += t < gs ? 0.f : v;
        }
        nu = sqrtf(hi ? s_hi : s_lo);
        nu_other = sqrtf(hi ? s_lo : s_hi);
        inv = nu > 0.f ? 1.f / nu : 0.f;
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] += part1_s[(mt * 16 + r) * 64 + lane];
        if (a.normalise) {
          nu = sqrtf(ss_s[0][l32] + ss_s[1][l32]);
          inv = nu > 0.f ? 1.f / nu : 0.f;
        }
      }
      uint32_t word[4] = {0u, 0u, 0u, 0u};
      float g2;
      if (hi) g2 = quantise_tile<(BITS < 4 ? BITS + 1 : 4)>(acc, inv, a.cb_hi, h, word);
      else g2 = quantise_tile<BITS>(acc, inv, a.cb, h, word);
      if (valid && h == 0) {
        uint32_t* dst = a.idx + oi * wpr + woff;
#pragma unroll
        for (int pl = 0; pl < BITS + (MIXED ? 1 : 0); ++pl)
          if (pl < BITS || hi) dst[pl] = word[pl];
        if (mt == 0 && a.norm != nullptr) {
          if (MIXED) {
            a.norm[2 * oi] = nu;  // tile 0 always belongs to instance hi
            a.norm[2 * oi + 1] = nu_other;
          } else {
            a.norm[oi] = nu;
          }
        }
      }
      if (PROD) {
        g2 += __shfl_xor(g2, 32);
        if (h == 0) g2_s[mt][l32] = g2;
#pragma unroll
        for (int k = 0; k < 4; ++k)
          *reinterpret_cast<f32x4*>(&e_s[l32 * E_LD + 32 * mt + 8 * k + 4 * h]) =
              f32x4{acc[4 * k], acc[4 * k + 1], acc[4 * k + 2], acc[4 * k + 3]};
      }
    }
    if (!PROD) {
      if (!MIXED) __syncthreads();  // the partial tiles and row sums are rewritten by the next block
      continue;
    }
    __syncthreads();

    // ---- U = (S Pi^T) E, same split; sign bits and gamma -----------------------------------
    floatx16 u;
#pragma unroll
    for (int r = 0; r < 16; ++r) u[r] = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const f32x4 ev = *reinterpret_cast<const f32x4*>(&e_s[l32 * E_LD + k0 + 4 * j]);
      u = __builtin_amdgcn_mfma_f32_32x32x2f32(sa[j].x, ev.x, u, 0, 0, 0);
      u = __builtin_amdgcn_mfma_f32_32x32x2f32(sa[j].y, ev.y, u, 0, 0, 0);
      u = __builtin_amdgcn_mfma_f32_32x32x2f32(sa[j].z, ev.z, u, 0, 0, 0);
      u = __builtin_amdgcn_mfma_f32_32x32x2f32(sa[j].w, ev.w, u, 0, 0, 0);
    }
    if (kh == 1) {
#pragma unroll
      for (int r = 0; r < 16; ++r) part2_s[(mt * 16 + r) * 64 + lane] = u[r];
    }
    __syncthreads();
    if (kh == 0) {
#pragma unroll
      for (int r = 0; r < 16; ++r) u[r] += part2_s[(mt * 16 + r) * 64 + lane];
      uint32_t nb[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        nb[k] = 0u;
#pragma unroll
        for (int r = 3; r >= 0; --r) nb[k] = nb[k] + nb[k] + (u[4 * k + r] >= 0.f ? 1u : 0u);
      }
      uint32_t w = (nb[0] | (nb[1] << 8) | (nb[2] << 16) | (nb[3] << 24)) << (4 * h);
      w |= (uint32_t)__shfl_xor((int)w, 32);
      if (valid && h == 0) {
        a.qjl[oi * 4 + mt] = w;
        if (mt == 0) {
          if (MIXED) {
            float g_hi = 0.f, g_lo = 0.f;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
              const float v = g2_s[t][l32];
              g_hi += t < gs ? v : 0.f;
              g_lo += t < gs ? 0.f : v;
            }
            a.gamma[2 * oi] = sqrtf(g_hi);
            a.gamma[2 * oi + 1] = sqrtf(g_lo);
          } else {
            a.gamma[oi] = sqrtf((g2_s[0][l32] + g2_s[1][l32]) + (g2_s[2][l32] + g2_s[3][l32]));
          }
        }
      }
    }
  }
}

// a workgroup takes one block up to this many workgroups; beyond that it loops over blocks,
// keeping its parameter slices in registers
constexpr int kSmallGrid = 1024;

template <int BITS, bool PROD, bool MIXED>
static hipError_t launch_in(const QuantSmallArgs& a, bool bf16, hipStream_t s) {
  const int64_t blocks = (a.n + 31) / 32;
  const dim3 grid((unsigned)(blocks < kSmallGrid ? blocks : kSmallGrid));
  if (bf16)
    hipLaunchKernelGGL((quant128_small_kernel<BITS, PROD, true, MIXED>), grid, dim3(512), 0, s, a);
  else
    hipLaunchKernelGGL((quant128_small_kernel<BITS, PROD, false, MIXED>), grid, dim3(512), 0, s, a);
  return hipGetLastError();
}

template <int BITS>
static hipError_t launch_bits(const QuantSmallArgs& a, bool prod, bool bf16, hipStream_t s) {
  if (a.gs_hi > 0) {
    if (BITS >= 4) return hipErrorInvalidValue;
    return prod ? launch_in<(BITS < 4 ? BITS : 0), true, true>(a, bf16, s)
                : launch_in<(BITS < 4 ? BITS : 0), false, true>(a, bf16, s);
  }
  return prod ? launch_in<BITS, true, false>(a, bf16, s) : launch_in<BITS, false, false>(a, bf16, s);
}

hipError_t launch_quant128_small(int bits, bool prod, bool bf16, const void* X, int64_t ldx, int64_t n,
                                 const float* Pi, const float* SPiT, uint32_t* idx, uint32_t* qjl,
                                 float* gamma, float* norm, const Codebook& cb, int gs_hi,
                                 const Codebook& cb_hi, hipStream_t s, int64_t out_first, int64_t out_step) {
  if (n == 0) return hipSuccess;
  if (gs_hi < 0 || gs_hi > 3 || (gs_hi > 0 && (cb_hi.bits != bits + 1 || norm == nullptr))) return hipErrorInvalidValue;
  QuantSmallArgs a;
  a.X = X; a.ldx = ldx; a.n = n; a.Pi = Pi; a.SPiT = SPiT; a.idx = idx; a.qjl = qjl; a.gamma = gamma;
  a.norm = norm; a.normalise = norm != nullptr; a.gs_hi = gs_hi; a.cb = cb; a.cb_hi = cb_hi;
  a.out_first = out_first; a.out_step = out_step;
  switch (bits) {
    case 0: return launch_bits<0>(a, prod, bf16, s);
    case 1: return launch_bits<1>(a, prod, bf16, s);
    case 2: return launch_bits<2>(a, prod, bf16, s);
    case 3: return launch_bits<3>(a, prod, bf16, s);
    case 4: return launch_bits<4>(a, prod, bf16, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace tq
