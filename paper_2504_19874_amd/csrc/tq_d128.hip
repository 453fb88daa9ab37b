// Fused kernels for head dimension d = 128 (KV-cache keys).  At this size the
// parameter matrices fit in the 160 KB LDS of a compute unit (Pi and S Pi^T,
// or Pi and S: 2 x 64 KB), so one 512-thread workgroup per CU loads them once
// and its 8 wavefronts then stream blocks of 32 vectors straight from HBM to
// registers to MFMA, with no further workgroup-level synchronisation.
//
// quant128:  Y^T = Pi X^T with the vector on the MFMA lane axis (see
//   tq_gemm.hip for the operand layout).  A lane loads one half (64 values) of
//   its own vector's row directly as the B operand: lane half h owns k in
//   [64h, 64h+64), which is just a permutation of the contraction order.  The
//   accumulator tile then holds y for 16 coordinates of that one vector per
//   lane; the epilogue turns it in place into the residual e = y - c[idx], and
//   those registers are *directly* the B operand of the second contraction
//   U^T = (S Pi^T) E^T (again only a permutation of k), so the residual never
//   leaves the register file.
//
// dequant128:  X~ = Y~ Pi + (kappa gamma Z) S with the vector on the MFMA row
//   axis (A operand decoded from the packed words in registers) and rows of
//   Pi / S as the B operand, read 16 bytes per lane so that the four output
//   tiles interleave columns 4l..4l+3: every output row is stored as one
//   contiguous 512-byte line.
#include "tq_d128_tile.h"

namespace tq {

constexpr int D = 128;
constexpr int PAD_LD = 132;  // padded row stride for 16-byte reads along k

struct Quant128Args {
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
  // two instances over a split of the rotated coordinates (MIXED, Sec. 4.3): coordinate groups
  // (= output tiles) [0, gs_hi) are quantised with BITS + 1 bits and cb_hi, each instance
  // normalised by the norm of its own rotated coordinates
  int gs_hi;
  Codebook cb_hi;
};

template <int BITS, bool PROD, bool BF16IN, bool MIXED>
__global__ __launch_bounds__(512) void quant128_kernel(const Quant128Args a) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  float* Pi_s = smem;
  float* Sp_s = smem + D * PAD_LD;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, h = lane >> 5;

  for (int p = 0; p < 8; ++p) {
    const int e4 = tid + 512 * p;  // 4096 float4 per matrix
    const int row = e4 >> 5, c4 = e4 & 31;
    *reinterpret_cast<float4*>(&Pi_s[row * PAD_LD + 4 * c4]) =
        *reinterpret_cast<const float4*>(a.Pi + row * D + 4 * c4);
    if (PROD)
      *reinterpret_cast<float4*>(&Sp_s[row * PAD_LD + 4 * c4]) =
          *reinterpret_cast<const float4*>(a.SPiT + row * D + 4 * c4);
  }
  __syncthreads();

  // fp32 MFMA and ordinary vector instructions do not overlap on this chip (a
  // wavefront doing v_fma while another does v_mfma_f32 takes the sum of both
  // times), so every vector instruction outside the contractions costs MFMA
  // time: the epilogues below are written for instruction count.
  constexpr int RAW = BF16IN ? 8 : 16;  // 16-byte loads per lane for one half row
  const int64_t n_blocks = (a.n + 31) / 32;
  const int64_t blk_stride = (int64_t)gridDim.x * 8;
  int64_t blk = (int64_t)blockIdx.x * 8 + wave;
  uint4 raw[RAW];
  auto load_raw = [&](int64_t b) {
    const int64_t i = b * 32 + l32;
    const bool ok = i < a.n;
    const char* src = reinterpret_cast<const char*>(a.X) +
                      ((ok ? i : 0) * a.ldx + 64 * h) * (BF16IN ? 2 : 4);
#pragma unroll
    for (int v = 0; v < RAW; ++v)
      raw[v] = ok ? *reinterpret_cast<const uint4*>(src + 16 * v) : make_uint4(0, 0, 0, 0);
  };
  if (blk < n_blocks) load_raw(blk);

  for (; blk < n_blocks; blk += blk_stride) {
    const int64_t i = blk * 32 + l32;
    const bool valid = i < a.n;
    float xb[64];
    if (BF16IN) {
#pragma unroll
      for (int v = 0; v < 8; ++v) {
        xb[8 * v + 0] = __uint_as_float(raw[v].x << 16); xb[8 * v + 1] = __uint_as_float(raw[v].x & 0xffff0000u);
        xb[8 * v + 2] = __uint_as_float(raw[v].y << 16); xb[8 * v + 3] = __uint_as_float(raw[v].y & 0xffff0000u);
        xb[8 * v + 4] = __uint_as_float(raw[v].z << 16); xb[8 * v + 5] = __uint_as_float(raw[v].z & 0xffff0000u);
        xb[8 * v + 6] = __uint_as_float(raw[v].w << 16); xb[8 * v + 7] = __uint_as_float(raw[v].w & 0xffff0000u);
      }
    } else {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        xb[4 * v] = __uint_as_float(raw[v].x); xb[4 * v + 1] = __uint_as_float(raw[v].y);
        xb[4 * v + 2] = __uint_as_float(raw[v].z); xb[4 * v + 3] = __uint_as_float(raw[v].w);
      }
    }
    float inv = 1.f, nu = 1.f;
    if (!MIXED && a.normalise) {
      float s0 = 0.f, s1 = 0.f;
#pragma unroll
      for (int k = 0; k < 64; k += 2) {
        s0 = fmaf(xb[k], xb[k], s0);
        s1 = fmaf(xb[k + 1], xb[k + 1], s1);
      }
      float ss = s0 + s1;
      ss += __shfl_xor(ss, 32);
      nu = sqrtf(ss);
      inv = nu > 0.f ? 1.f / nu : 0.f;
    }

    floatx16 acc[4];
    {
      // operands of step k4+1 are read from LDS before the MFMAs of step k4 issue;
      // the very first MFMA of each tile takes a zero C operand instead of a cleared register
      const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      float4 av[4], nx[4];
#pragma unroll
      for (int t = 0; t < 4; ++t)
        av[t] = *reinterpret_cast<const float4*>(&Pi_s[(32 * t + l32) * PAD_LD + 64 * h]);
#pragma unroll
      for (int k4 = 0; k4 < 16; ++k4) {
        if (k4 + 1 < 16) {
#pragma unroll
          for (int t = 0; t < 4; ++t)
            nx[t] = *reinterpret_cast<const float4*>(&Pi_s[(32 * t + l32) * PAD_LD + 64 * h + 4 * (k4 + 1)]);
        }
#pragma unroll
        for (int t = 0; t < 4; ++t)
          acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[t].x, xb[4 * k4 + 0], k4 == 0 ? zero : acc[t], 0, 0, 0);
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[t].y, xb[4 * k4 + 1], acc[t], 0, 0, 0);
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[t].z, xb[4 * k4 + 2], acc[t], 0, 0, 0);
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[t].w, xb[4 * k4 + 3], acc[t], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);  // bounds how far LDS reads are hoisted (register pressure)
#pragma unroll
        for (int t = 0; t < 4; ++t) av[t] = nx[t];
      }
    }
    // the next block's rows travel from HBM while this block is finished
    if (blk + blk_stride < n_blocks) load_raw(blk + blk_stride);

    float g2 = 0.f, g2_hi = 0.f;
    if (MIXED) {
      // norms of the two instances from the rotated coordinates, then tile by tile with the
      // instance's own codebook and bit count
      const int gs = a.gs_hi;
      float s_hi = 0.f, s_lo = 0.f;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          s0 = fmaf(acc[t][r], acc[t][r], s0);
          s1 = fmaf(acc[t][r + 1], acc[t][r + 1], s1);
        }
        const float ts = s0 + s1;
        s_hi += t < gs ? ts : 0.f;
        s_lo += t < gs ? 0.f : ts;
      }
      s_hi += __shfl_xor(s_hi, 32);
      s_lo += __shfl_xor(s_lo, 32);
      const float nu_hi = sqrtf(s_hi), nu_lo = sqrtf(s_lo);
      const float inv_hi = nu_hi > 0.f ? 1.f / nu_hi : 0.f, inv_lo = nu_lo > 0.f ? 1.f / nu_lo : 0.f;
      const int wpr = 4 * BITS + gs;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        uint32_t wd[4] = {0u, 0u, 0u, 0u};
        const bool thi = t < gs;  // uniform
        if (thi) g2_hi += quantise_tile<(BITS < 4 ? BITS + 1 : 4)>(acc[t], inv_hi, a.cb_hi, h, wd);
        else g2 += quantise_tile<BITS>(acc[t], inv_lo, a.cb, h, wd);
        // both half-waves hold the merged words; half t / 2 stores them
        if (valid && h == (t >> 1)) {
          uint32_t* dst = a.idx + i * wpr + (thi ? t * (BITS + 1) : gs * (BITS + 1) + (t - gs) * BITS);
#pragma unroll
          for (int pl = 0; pl < BITS + 1; ++pl)
            if (pl < BITS || thi) dst[pl] = wd[pl];
        }
      }
      if (valid && h == 0) {
        a.norm[2 * i] = nu_hi;
        a.norm[2 * i + 1] = nu_lo;
      }
    } else {
    // nearest centroid, packing, residual (in place).  Bit p of the bucket number is the XOR
    // of the compare masks at positions k = 2^p - 1 (mod 2^p); a 4-bit nibble of a plane is
    // built by shift-and-add-carry, most significant element first.
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      uint32_t nib[4][BITS > 0 ? BITS : 1];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
#pragma unroll
        for (int pl = 0; pl < (BITS > 0 ? BITS : 1); ++pl) nib[k][pl] = 0u;
#pragma unroll
        for (int r = 3; r >= 0; --r) {
          const float y = acc[t][4 * k + r] * inv;
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
          acc[t][4 * k + r] = e;
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
        // both half-waves hold the merged word; half t / 2 stores it (coordinate group t)
        if (valid && h == (t >> 1)) a.idx[i * (4 * BITS) + t * BITS + pl] = w;
      }
    }
    if (valid && h == 0 && a.norm != nullptr) a.norm[i] = nu;

    }
    if (PROD) {
      g2 += __shfl_xor(g2, 32);
      if (MIXED) g2_hi += __shfl_xor(g2_hi, 32);
      floatx16 u[4];
      // register 4*ke + r of tile te holds e_j with j = 32 te + 8 ke + 4 h + r
      {
        const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        float4 av[4], nx[4];
#pragma unroll
        for (int t = 0; t < 4; ++t)
          av[t] = *reinterpret_cast<const float4*>(&Sp_s[(32 * t + l32) * PAD_LD + 4 * h]);
#pragma unroll
        for (int st = 0; st < 16; ++st) {
          const int te = st >> 2, ke = st & 3;
          if (st + 1 < 16) {
            const int te1 = (st + 1) >> 2, ke1 = (st + 1) & 3;
#pragma unroll
            for (int t = 0; t < 4; ++t)
              nx[t] = *reinterpret_cast<const float4*>(
                  &Sp_s[(32 * t + l32) * PAD_LD + 32 * te1 + 8 * ke1 + 4 * h]);
          }
#pragma unroll
          for (int t = 0; t < 4; ++t)
            u[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[t].x, acc[te][4 * ke + 0], st == 0 ? zero : u[t], 0, 0, 0);
#pragma unroll
          for (int t = 0; t < 4; ++t) u[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[t].y, acc[te][4 * ke + 1], u[t], 0, 0, 0);
#pragma unroll
          for (int t = 0; t < 4; ++t) u[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[t].z, acc[te][4 * ke + 2], u[t], 0, 0, 0);
#pragma unroll
          for (int t = 0; t < 4; ++t) u[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[t].w, acc[te][4 * ke + 3], u[t], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int t = 0; t < 4; ++t) av[t] = nx[t];
        }
      }
      uint32_t sw[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        uint32_t nib[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          nib[k] = 0u;
#pragma unroll
          for (int r = 3; r >= 0; --r) nib[k] = nib[k] + nib[k] + (u[t][4 * k + r] >= 0.f ? 1u : 0u);
          __builtin_amdgcn_sched_barrier(0);
        }
        const uint32_t w = (nib[0] | (nib[1] << 8) | (nib[2] << 16) | (nib[3] << 24)) << (4 * h);
        sw[t] = w | (uint32_t)__shfl_xor((int)w, 32);
      }
      if (valid) {
        uint32_t* dst = a.qjl + i * 4 + 2 * h;
        dst[0] = h ? sw[2] : sw[0];
        dst[1] = h ? sw[3] : sw[1];
        if (h == 0) {
          if (MIXED) {
            a.gamma[2 * i] = sqrtf(g2_hi);
            a.gamma[2 * i + 1] = sqrtf(g2);
          } else {
            a.gamma[i] = sqrtf(g2);
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
struct Dequant128Args {
  const uint32_t* idx;
  const uint32_t* qjl;
  const float* gamma;
  const float* norm;
  const float* Pi;
  const float* S;
  float* out;
  int64_t ldo;
  int64_t n;
  float kappa;
  Codebook cb;
  // two instances over a split of the rotated coordinates (MIXED): groups [0, gs_hi) belong to
  // instance hi with BITS + 1 planes, codebook cb_hi and sketch scale kappa_hi
  int gs_hi;
  float kappa_hi;
  Codebook cb_hi;
};

template <int BITS, bool PROD, bool MIXED>
__global__ __launch_bounds__(512) void dequant128_kernel(const Dequant128Args a) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  __shared__ float cent_s[16];
  __shared__ float cent_hi_s[32];
  float* Pi_s = smem;          // [128][128], rows read contiguously
  float* S_s = smem + D * D;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, h = lane >> 5;
  if (tid < 16) cent_s[tid] = a.cb.c[tid];
  if (MIXED && tid < 16) cent_hi_s[tid] = a.cb_hi.c[tid];
  const int gs = MIXED ? a.gs_hi : 0;
  for (int p = 0; p < 8; ++p) {
    const int e4 = tid + 512 * p;
    reinterpret_cast<float4*>(Pi_s)[e4] = reinterpret_cast<const float4*>(a.Pi)[e4];
    if (PROD) reinterpret_cast<float4*>(S_s)[e4] = reinterpret_cast<const float4*>(a.S)[e4];
  }
  __syncthreads();

  const int64_t n_blocks = (a.n + 31) / 32;
  for (int64_t blk = (int64_t)blockIdx.x * 8 + wave; blk < n_blocks; blk += (int64_t)gridDim.x * 8) {
    const int64_t i = blk * 32 + l32;
    const bool valid = i < a.n;
    const int64_t row = valid ? i : 0;
    // per-instance scalars: index 1 = instance hi (MIXED only), index 0 = the (only / lo) instance
    float nu[2], kg[2] = {0.f, 0.f};
    if (MIXED) {
      nu[1] = valid ? a.norm[2 * row] : 0.f;
      nu[0] = valid ? a.norm[2 * row + 1] : 0.f;
      if (PROD) {
        kg[1] = nu[1] * a.kappa_hi * a.gamma[2 * row];
        kg[0] = nu[0] * a.kappa * a.gamma[2 * row + 1];
      }
    } else {
      nu[0] = nu[1] = (valid && a.norm != nullptr) ? a.norm[row] : (valid ? 1.f : 0.f);
      if (PROD) kg[0] = kg[1] = nu[0] * a.kappa * a.gamma[row];
    }
    floatx16 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

    if (BITS > 0 || MIXED) {
      // plane words of each group, shifted to this half's 16 coordinates; a group of instance lo
      // has no plane BITS (left zero), so one decode serves both
      constexpr int NP = BITS + (MIXED ? 1 : 0);
      constexpr int BD = BITS > 0 ? BITS : 1;
      uint32_t wg[4][NP > 0 ? NP : 1];
      if (MIXED) {
        const uint32_t* src = a.idx + row * (4 * BITS + gs);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int base = g < gs ? g * (BITS + 1) : gs * (BITS + 1) + (g - gs) * BITS;
#pragma unroll
          for (int pl = 0; pl < NP; ++pl) wg[g][pl] = (pl < BITS || g < gs) ? src[base + pl] >> (16 * h) : 0u;
        }
      } else {
        const uint32_t* src = a.idx + row * (4 * BITS);
#pragma unroll
        for (int v = 0; v < BITS; ++v) {
          const uint4 t4 = *reinterpret_cast<const uint4*>(src + 4 * v);
          const uint32_t w4[4] = {t4.x, t4.y, t4.z, t4.w};
#pragma unroll
          for (int q = 0; q < 4; ++q) wg[(4 * v + q) / BD][(4 * v + q) % BD] = w4[q] >> (16 * h);
        }
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const bool ghi = MIXED && g < gs;  // uniform
        const float* const tab = ghi ? cent_hi_s : cent_s;
        const float nug = ghi ? nu[1] : nu[0];
#pragma unroll
        for (int s = 0; s < 16; ++s) {
          uint32_t code = 0u;
#pragma unroll
          for (int pl = 0; pl < NP; ++pl) code |= ((wg[g][pl] >> s) & 1u) << pl;
          const float av = nug * tab[code];
          const float4 bv = *reinterpret_cast<const float4*>(&Pi_s[(32 * g + 16 * h + s) * D + 4 * l32]);
          acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv.x, acc[0], 0, 0, 0);
          acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv.y, acc[1], 0, 0, 0);
          acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv.z, acc[2], 0, 0, 0);
          acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv.w, acc[3], 0, 0, 0);
          if ((s & 3) == 3) __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    if (PROD) {
      const uint4 t4 = *reinterpret_cast<const uint4*>(a.qjl + row * 4);
      const uint32_t z[4] = {t4.x >> (16 * h), t4.y >> (16 * h), t4.z >> (16 * h), t4.w >> (16 * h)};
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float kgg = (MIXED && g < gs) ? kg[1] : kg[0];
#pragma unroll
        for (int s = 0; s < 16; ++s) {
          const float av = ((z[g] >> s) & 1u) ? kgg : -kgg;
          const float4 bv = *reinterpret_cast<const float4*>(&S_s[(32 * g + 16 * h + s) * D + 4 * l32]);
          acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv.x, acc[0], 0, 0, 0);
          acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv.y, acc[1], 0, 0, 0);
          acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv.z, acc[2], 0, 0, 0);
          acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv.w, acc[3], 0, 0, 0);
          if ((s & 3) == 3) __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    // D[row][col]: register 4k+r of a lane is row 8k + 4h + r; tile t, lane column l32 is
    // output column 4*l32 + t: one float4 per row per lane, 512 contiguous bytes per row
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int64_t orow = blk * 32 + 8 * k + 4 * h + r;
        if (orow < a.n)
          *reinterpret_cast<float4*>(a.out + orow * a.ldo + 4 * l32) =
              make_float4(acc[0][4 * k + r], acc[1][4 * k + r], acc[2][4 * k + r], acc[3][4 * k + r]);
      }
  }
}

// ------------------------------- launchers -------------------------------

static int grid_128(int64_t n) {
  const int64_t blocks = (n + 31) / 32;
  int64_t g = (blocks + 7) / 8;
  const int64_t cus = device_cu_count();
  if (g > cus) g = cus;  // one workgroup per compute unit
  return (int)(g < 1 ? 1 : g);
}

template <int BITS, bool PROD, bool BF16IN, bool MIXED>
static hipError_t launch_q(const Quant128Args& a, hipStream_t s) {
  const size_t smem = (size_t)(PROD ? 2 : 1) * D * PAD_LD * sizeof(float);
  static LdsLimit lds_limit;  // per instantiation: the limit is raised once per device
  if (const hipError_t e = raise_lds_limit(lds_limit, reinterpret_cast<const void*>(&quant128_kernel<BITS, PROD, BF16IN, MIXED>), (int)smem); e != hipSuccess) return e;
  hipLaunchKernelGGL((quant128_kernel<BITS, PROD, BF16IN, MIXED>), dim3(grid_128(a.n)), dim3(512), smem, s, a);
  return hipGetLastError();
}

template <int BITS, bool MIXED>
static hipError_t launch_q_in(const Quant128Args& a, bool prod, bool bf16, hipStream_t s) {
  if (prod) return bf16 ? launch_q<BITS, true, true, MIXED>(a, s) : launch_q<BITS, true, false, MIXED>(a, s);
  return bf16 ? launch_q<BITS, false, true, MIXED>(a, s) : launch_q<BITS, false, false, MIXED>(a, s);
}

template <int BITS>
static hipError_t launch_q_bits(const Quant128Args& a, bool prod, bool bf16, hipStream_t s) {
  if (a.gs_hi > 0) {
    if (BITS >= 4) return hipErrorInvalidValue;
    return launch_q_in<(BITS < 4 ? BITS : 0), true>(a, prod, bf16, s);
  }
  return launch_q_in<BITS, false>(a, prod, bf16, s);
}

hipError_t launch_quant128(int bits, bool prod, bool bf16, const void* X, int64_t ldx, int64_t n,
                           const float* Pi, const float* SPiT, uint32_t* idx, uint32_t* qjl, float* gamma,
                           float* norm, const Codebook& cb, int gs_hi, const Codebook& cb_hi, hipStream_t s) {
  if (n == 0) return hipSuccess;
  if (gs_hi < 0 || gs_hi > 3 || (gs_hi > 0 && (cb_hi.bits != bits + 1 || norm == nullptr))) return hipErrorInvalidValue;
  // up to about one block of 32 vectors per wavefront slot of the chip, a workgroup per block
  // (tq_d128_small.hip) is the shorter chain; beyond that the streaming kernel below wins
  if (n <= kSmallQuantRows)
    return launch_quant128_small(bits, prod, bf16, X, ldx, n, Pi, SPiT, idx, qjl, gamma, norm, cb, gs_hi, cb_hi, s);
  Quant128Args a;
  a.X = X; a.ldx = ldx; a.n = n; a.Pi = Pi; a.SPiT = SPiT; a.idx = idx; a.qjl = qjl; a.gamma = gamma;
  a.norm = norm; a.normalise = norm != nullptr; a.cb = cb; a.gs_hi = gs_hi; a.cb_hi = cb_hi;
  switch (bits) {
    case 0: return launch_q_bits<0>(a, prod, bf16, s);
    case 1: return launch_q_bits<1>(a, prod, bf16, s);
    case 2: return launch_q_bits<2>(a, prod, bf16, s);
    case 3: return launch_q_bits<3>(a, prod, bf16, s);
    case 4: return launch_q_bits<4>(a, prod, bf16, s);
    default: return hipErrorInvalidValue;
  }
}

template <int BITS, bool PROD, bool MIXED>
static hipError_t launch_dm(const Dequant128Args& a, hipStream_t s) {
  const size_t smem = (size_t)(PROD ? 2 : 1) * D * D * sizeof(float);
  static LdsLimit lds_limit;  // per instantiation: the limit is raised once per device
  if (const hipError_t e = raise_lds_limit(lds_limit, reinterpret_cast<const void*>(&dequant128_kernel<BITS, PROD, MIXED>), (int)smem); e != hipSuccess) return e;
  hipLaunchKernelGGL((dequant128_kernel<BITS, PROD, MIXED>), dim3(grid_128(a.n)), dim3(512), smem, s, a);
  return hipGetLastError();
}

template <int BITS, bool PROD>
static hipError_t launch_d(const Dequant128Args& a, hipStream_t s) {
  if (a.gs_hi > 0) {
    if (BITS >= 4) return hipErrorInvalidValue;
    return launch_dm<(BITS < 4 ? BITS : 0), PROD, true>(a, s);
  }
  return launch_dm<BITS, PROD, false>(a, s);
}

hipError_t launch_dequant128(int bits, bool prod, const uint32_t* idx, const uint32_t* qjl,
                             const float* gamma, const float* norm, const float* Pi, const float* S,
                             float* out, int64_t ldo, int64_t n, float kappa, const Codebook& cb,
                             int gs_hi, float kappa_hi, const Codebook& cb_hi, hipStream_t s) {
  if (n == 0) return hipSuccess;
  if (gs_hi < 0 || gs_hi > 3 || (gs_hi > 0 && (cb_hi.bits != bits + 1 || norm == nullptr))) return hipErrorInvalidValue;
  // a few blocks of 32 vectors: one workgroup per block is the shorter chain (tq_d128_small_dq.hip)
  if (n <= kSmallDequantRows)
    return launch_dequant128_small(bits, prod, idx, qjl, gamma, norm, Pi, S, out, ldo, n, kappa, cb, gs_hi, kappa_hi,
                                   cb_hi, s);
  Dequant128Args a;
  a.idx = idx; a.qjl = qjl; a.gamma = gamma; a.norm = norm; a.Pi = Pi; a.S = S; a.out = out; a.ldo = ldo;
  a.n = n; a.kappa = kappa; a.cb = cb; a.gs_hi = gs_hi; a.kappa_hi = kappa_hi; a.cb_hi = cb_hi;
  switch (bits) {
    case 0: return prod ? launch_d<0, true>(a, s) : launch_d<0, false>(a, s);
    case 1: return prod ? launch_d<1, true>(a, s) : launch_d<1, false>(a, s);
    case 2: return prod ? launch_d<2, true>(a, s) : launch_d<2, false>(a, s);
    case 3: return prod ? launch_d<3, true>(a, s) : launch_d<3, false>(a, s);
    case 4: return prod ? launch_d<4, true>(a, s) : launch_d<4, false>(a, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace tq
