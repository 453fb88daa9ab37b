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
#include "tq_internal.h"

namespace tq {

typedef float floatx16 __attribute__((ext_vector_type(16)));
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
  int normalise;
  Codebook cb;
};

constexpr int E_LD = 132;  // padded row stride of the residual tile in LDS

template <int BITS, bool PROD, bool BF16IN>
__global__ __launch_bounds__(512) void quant128_small_kernel(const QuantSmallArgs a) {
  __shared__ __attribute__((aligned(16))) float part_s[4 * 16 * 64];  // upper-half partial tiles [tile][register][lane]
  __shared__ __attribute__((aligned(16))) float e_s[32 * E_LD];       // residual [vector][coordinate]
  __shared__ float ss_s[2][32];                                       // partial sums of squares of x
  __shared__ float g2_s[4][32];                                       // partial squared residual norms
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, h = lane >> 5;
  const int mt = wave & 3, kh = wave >> 2;
  const int64_t i = (int64_t)blockIdx.x * 32 + l32;
  const bool valid = i < a.n;
  const int k0 = 64 * h + 32 * kh;  // first contraction index of this lane

  // ---- everything this wavefront reads from memory, requested up front ------------------
  f32x4 pa[8], sa[8];
  {
    const float* prow = a.Pi + (32 * mt + l32) * 128 + k0;
#pragma unroll
    for (int j = 0; j < 8; ++j) pa[j] = *reinterpret_cast<const f32x4*>(prow + 4 * j);
  }
  float xb[32];
  {
    const char* src = reinterpret_cast<const char*>(a.X) + ((valid ? i : a.n - 1) * a.ldx + k0) * (BF16IN ? 2 : 4);
    if (BF16IN) {
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const u32x4 r = *reinterpret_cast<const u32x4*>(src + 16 * v);
        xb[8 * v + 0] = __uint_as_float(r.x << 16); xb[8 * v + 1] = __uint_as_float(r.x & 0xffff0000u);
        xb[8 * v + 2] = __uint_as_float(r.y << 16); xb[8 * v + 3] = __uint_as_float(r.y & 0xffff0000u);
        xb[8 * v + 4] = __uint_as_float(r.z << 16); xb[8 * v + 5] = __uint_as_float(r.z & 0xffff0000u);
        xb[8 * v + 6] = __uint_as_float(r.w << 16); xb[8 * v + 7] = __uint_as_float(r.w & 0xffff0000u);
      }
    } else {
#pragma unroll
      for (int v = 0; v < 8; ++v) {
        const f32x4 r = *reinterpret_cast<const f32x4*>(src + 16 * v);
        xb[4 * v] = r.x; xb[4 * v + 1] = r.y; xb[4 * v + 2] = r.z; xb[4 * v + 3] = r.w;
      }
    }
  }
  if (PROD) {
    const float* srow = a.SPiT + (32 * mt + l32) * 128 + k0;
#pragma unroll
    for (int j = 0; j < 8; ++j) sa[j] = *reinterpret_cast<const f32x4*>(srow + 4 * j);
  }

  // ---- norm: tile-0 wavefronts add up their quarter of each row -----------------------------
  if (a.normalise && mt == 0) {
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

  // ---- Y = Pi X: this wavefront's tile over its half of k ------------------------------------
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
    for (int r = 0; r < 16; ++r) part_s[(mt * 16 + r) * 64 + lane] = acc[r];
  }
  __syncthreads();

  float nu = 1.f;
  if (kh == 0) {
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] += part_s[(mt * 16 + r) * 64 + lane];
    float inv = 1.f;
    if (a.normalise) {
      nu = sqrtf(ss_s[0][l32] + ss_s[1][l32]);
      inv = nu > 0.f ? 1.f / nu : 0.f;
    }
    // nearest centroid, packing, residual (in place).  Bit p of the bucket number is the XOR
    // of the compare masks at positions k = 2^p - 1 (mod 2^p); a 4-bit nibble of a plane is
    // built by shift-and-add-carry, most significant element first.
    float g2 = 0.f;
    uint32_t nib[4][BITS > 0 ? BITS : 1];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
#pragma unroll
      for (int pl = 0; pl < (BITS > 0 ? BITS : 1); ++pl) nib[k][pl] = 0u;
#pragma unroll
      for (int r = 3; r >= 0; --r) {
        const float y = acc[4 * k + r] * inv;
        float yt = a.cb.c[0];
        bool bit[BITS > 0 ? BITS : 1];
#pragma unroll
        for (int pl = 0; pl < (BITS > 0 ? BITS : 1); ++pl) bit[pl] = false;
#pragma unroll
        for (int j = 0; j < (1 << BITS) - 1; ++j) {
          const bool ge = y >= a.cb.t[j];
          yt = ge ? a.cb.c[j + 1] : yt;
#pragma unroll
          for (int pl = 0; pl < BITS; ++pl)
            if ((j & ((1 << pl) - 1)) == (1 << pl) - 1) bit[pl] = bit[pl] != ge;
        }
        float e = y - yt;
        asm volatile("" : "+v"(e));  // keep the residual here: sunk later it would need the masks again
        g2 = fmaf(e, e, g2);
        acc[4 * k + r] = e;
#pragma unroll
        for (int pl = 0; pl < BITS; ++pl) {
          nib[k][pl] = nib[k][pl] + nib[k][pl] + (bit[pl] ? 1u : 0u);
          asm volatile("" : "+v"(nib[k][pl]));  // consume this element's masks now (scalar registers)
        }
      }
    }
#pragma unroll
    for (int pl = 0; pl < BITS; ++pl) {
      uint32_t w = (nib[0][pl] | (nib[1][pl] << 8) | (nib[2][pl] << 16) | (nib[3][pl] << 24)) << (4 * h);
      w |= (uint32_t)__shfl_xor((int)w, 32);
      if (valid && h == 0) a.idx[i * (4 * BITS) + mt * BITS + pl] = w;
    }
    if (valid && h == 0 && mt == 0 && a.norm != nullptr) a.norm[i] = nu;
    if (PROD) {
      g2 += __shfl_xor(g2, 32);
      if (h == 0) g2_s[mt][l32] = g2;
#pragma unroll
      for (int k = 0; k < 4; ++k)
        *reinterpret_cast<f32x4*>(&e_s[l32 * E_LD + 32 * mt + 8 * k + 4 * h]) =
            f32x4{acc[4 * k], acc[4 * k + 1], acc[4 * k + 2], acc[4 * k + 3]};
    }
  }
  if (!PROD) return;
  __syncthreads();

  // ---- U = (S Pi^T) E, same split; sign bits and gamma ---------------------------------------
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
    for (int r = 0; r < 16; ++r) part_s[(mt * 16 + r) * 64 + lane] = u[r];
  }
  __syncthreads();
  if (kh == 0) {
#pragma unroll
    for (int r = 0; r < 16; ++r) u[r] += part_s[(mt * 16 + r) * 64 + lane];
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
      a.qjl[i * 4 + mt] = w;
      if (mt == 0) a.gamma[i] = sqrtf((g2_s[0][l32] + g2_s[1][l32]) + (g2_s[2][l32] + g2_s[3][l32]));
    }
  }
}

template <int BITS, bool PROD>
static hipError_t launch_in(const QuantSmallArgs& a, bool bf16, hipStream_t s) {
  const dim3 grid((unsigned)((a.n + 31) / 32));
  if (bf16)
    hipLaunchKernelGGL((quant128_small_kernel<BITS, PROD, true>), grid, dim3(512), 0, s, a);
  else
    hipLaunchKernelGGL((quant128_small_kernel<BITS, PROD, false>), grid, dim3(512), 0, s, a);
  return hipGetLastError();
}

template <int BITS>
static hipError_t launch_bits(const QuantSmallArgs& a, bool prod, bool bf16, hipStream_t s) {
  return prod ? launch_in<BITS, true>(a, bf16, s) : launch_in<BITS, false>(a, bf16, s);
}

hipError_t launch_quant128_small(int bits, bool prod, bool bf16, const void* X, int64_t ldx, int64_t n,
                                 const float* Pi, const float* SPiT, uint32_t* idx, uint32_t* qjl,
                                 float* gamma, float* norm, const Codebook& cb, hipStream_t s) {
  if (n == 0) return hipSuccess;
  QuantSmallArgs a;
  a.X = X; a.ldx = ldx; a.n = n; a.Pi = Pi; a.SPiT = SPiT; a.idx = idx; a.qjl = qjl; a.gamma = gamma;
  a.norm = norm; a.normalise = norm != nullptr; a.cb = cb;
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
