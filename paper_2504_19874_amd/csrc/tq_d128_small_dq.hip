// Dequantisation at d = 128 for a small number of vectors (the counterpart of
// tq_d128_small.hip): one workgroup of 8 wavefronts per block of 32 vectors.
//
// x~ = sum_j y~'_j Pi[j][:] + sum_j z'_j S[j][:]  with y~'_j = nu c[idx_j] and
// z'_j = +-nu kappa gamma: 256 (prod) or 128 (mse) terms per vector.  Wavefront w
// takes a slice of them for all 128 output columns: prod: coordinate group
// w % 4 (32 coordinates) of part w / 4 (0: codebook part against Pi, 1: sign
// part against S); mse: half w / 4 (16 coordinates) of group w % 4.  Its rows of
// Pi / S come straight from L2, 16 bytes per lane so that the four output tiles
// interleave columns 4l..4l+3 (as in dequant128_kernel) and are requested
// before anything else.  The 8 partial results are added through LDS in two
// steps; wavefront 0 stores the rows, 512 contiguous bytes each.
#include "tq_internal.h"

namespace tq {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct DequantSmallArgs {
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
  int gs_hi;  // two instances (MIXED): coordinate groups [0, gs_hi) belong to instance hi
  float kappa_hi;
  Codebook cb_hi;
};

template <int BITS, bool PROD, bool MIXED>
__global__ __launch_bounds__(512) void dequant128_small_kernel(const DequantSmallArgs a) {
  extern __shared__ __attribute__((aligned(16))) float part_s[];  // 64 KB: [slot][tile * 16 + register][lane]
  __shared__ float cent_s[16];
  __shared__ float cent_hi_s[16];
  constexpr int NP = BITS + (MIXED ? 1 : 0);
  constexpr int STEPS = PROD ? 16 : 8;  // MFMA k-steps (2 coordinates each) of this wavefront's slice
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, h = lane >> 5;
  const int g = wave & 3, part = wave >> 2;
  const int gs = MIXED ? a.gs_hi : 0;
  const bool ghi = MIXED && g < gs;  // uniform
  if (tid < 16) {
    cent_s[tid] = a.cb.c[tid];
    cent_hi_s[tid] = MIXED ? a.cb_hi.c[tid] : 0.f;
  }

  // first coordinate of this lane's run: prod: 32 g + 16 h + s; mse: 32 g + 16 part + 8 h + s
  const int j0 = PROD ? 32 * g + 16 * h : 32 * g + 16 * part + 8 * h;
  constexpr int RUN = PROD ? 16 : 8;
  const bool sign_part = PROD && part == 1;
  f32x4 bv[RUN];
  {
    const float* rows = (sign_part ? a.S : a.Pi) + j0 * 128 + 4 * l32;
#pragma unroll
    for (int s = 0; s < RUN; ++s) bv[s] = *reinterpret_cast<const f32x4*>(rows + s * 128);
  }
  const int64_t i = (int64_t)blockIdx.x * 32 + l32;
  const bool valid = i < a.n;
  const int64_t row = valid ? i : a.n - 1;
  float nu, kg = 0.f;
  if (MIXED) {
    nu = a.norm[2 * row + (ghi ? 0 : 1)];
    if (PROD) kg = nu * (ghi ? a.kappa_hi : a.kappa) * a.gamma[2 * row + (ghi ? 0 : 1)];
  } else {
    nu = a.norm != nullptr ? a.norm[row] : 1.f;
    if (PROD) kg = nu * a.kappa * a.gamma[row];
  }
  // the bits of this lane's run, one word per plane (plane BITS exists for instance hi only)
  uint32_t w[NP > 0 ? NP : 1];
  const int shift = PROD ? 16 * h : 16 * part + 8 * h;
  if (sign_part) {
    w[0] = a.qjl[row * 4 + g] >> shift;
  } else {
    const int wpr = MIXED ? 4 * BITS + gs : 4 * BITS;
    const int woff = MIXED ? (g < gs ? g * (BITS + 1) : gs * (BITS + 1) + (g - gs) * BITS) : g * BITS;
#pragma unroll
    for (int pl = 0; pl < NP; ++pl) w[pl] = (pl < BITS || ghi) ? a.idx[row * wpr + woff + pl] >> shift : 0u;
  }
  __syncthreads();  // centroid tables

  floatx16 acc[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
  const float* const tab = ghi ? cent_hi_s : cent_s;
  if (sign_part || NP > 0) {
#pragma unroll
    for (int s = 0; s < RUN; ++s) {
      float av;
      if (sign_part) {
        av = ((w[0] >> s) & 1u) ? kg : -kg;
      } else {
        uint32_t code = 0u;
#pragma unroll
        for (int pl = 0; pl < NP; ++pl) code |= ((w[pl] >> s) & 1u) << pl;
        av = nu * tab[code];
      }
      if (!valid) av = 0.f;
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv[s].x, acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv[s].y, acc[1], 0, 0, 0);
      acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv[s].z, acc[2], 0, 0, 0);
      acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv[s].w, acc[3], 0, 0, 0);
    }
  }

  // ---- 8 partial results -> 4 -> 1 ---------------------------------------------------------
  auto put = [&](int slot) {
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) part_s[(slot * 64 + t * 16 + r) * 64 + lane] = acc[t][r];
  };
  auto add = [&](int slot) {
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[t][r] += part_s[(slot * 64 + t * 16 + r) * 64 + lane];
  };
  if (wave >= 4) put(wave - 4);
  __syncthreads();
  if (wave < 4) add(wave);
  __syncthreads();
  if (wave >= 1 && wave < 4) put(wave);
  __syncthreads();
  if (wave == 0) {
    add(1);
    add(2);
    add(3);
    // D[row][col]: register 4k+r of a lane is row 8k + 4h + r; tile t, lane column l32 is output
    // column 4*l32 + t: one 16-byte piece per row per lane, 512 contiguous bytes per row
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int64_t orow = (int64_t)blockIdx.x * 32 + 8 * k + 4 * h + r;
        if (orow < a.n)
          *reinterpret_cast<f32x4*>(a.out + orow * a.ldo + 4 * l32) =
              f32x4{acc[0][4 * k + r], acc[1][4 * k + r], acc[2][4 * k + r], acc[3][4 * k + r]};
      }
  }
}

template <int BITS, bool PROD, bool MIXED>
static hipError_t launch_one(const DequantSmallArgs& a, hipStream_t s) {
  constexpr int lds = 4 * 64 * 64 * (int)sizeof(float);  // with the static tables just above the 64 KB default limit
  static LdsLimit lds_limit;  // per instantiation: the limit is raised once per device
  if (const hipError_t e = raise_lds_limit(lds_limit, reinterpret_cast<const void*>(&dequant128_small_kernel<BITS, PROD, MIXED>), lds); e != hipSuccess) return e;
  hipLaunchKernelGGL((dequant128_small_kernel<BITS, PROD, MIXED>), dim3((unsigned)((a.n + 31) / 32)), dim3(512), lds, s, a);
  return hipGetLastError();
}

template <int BITS>
static hipError_t launch_bits(const DequantSmallArgs& a, bool prod, hipStream_t s) {
  if (a.gs_hi > 0) {
    if (BITS >= 4) return hipErrorInvalidValue;
    return prod ? launch_one<(BITS < 4 ? BITS : 0), true, true>(a, s) : launch_one<(BITS < 4 ? BITS : 0), false, true>(a, s);
  }
  return prod ? launch_one<BITS, true, false>(a, s) : launch_one<BITS, false, false>(a, s);
}

hipError_t launch_dequant128_small(int bits, bool prod, const uint32_t* idx, const uint32_t* qjl,
                                   const float* gamma, const float* norm, const float* Pi, const float* S,
                                   float* out, int64_t ldo, int64_t n, float kappa, const Codebook& cb,
                                   int gs_hi, float kappa_hi, const Codebook& cb_hi, hipStream_t s) {
  if (n == 0) return hipSuccess;
  DequantSmallArgs a;
  a.idx = idx; a.qjl = qjl; a.gamma = gamma; a.norm = norm; a.Pi = Pi; a.S = S; a.out = out; a.ldo = ldo;
  a.n = n; a.kappa = kappa; a.cb = cb; a.gs_hi = gs_hi; a.kappa_hi = kappa_hi; a.cb_hi = cb_hi;
  switch (bits) {
    case 0: return launch_bits<0>(a, prod, s);
    case 1: return launch_bits<1>(a, prod, s);
    case 2: return launch_bits<2>(a, prod, s);
    case 3: return launch_bits<3>(a, prod, s);
    case 4: return launch_bits<4>(a, prod, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace tq
