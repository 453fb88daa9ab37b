// DeQuant (Alg. 1 / Alg. 2) at d = 128 for large batches, on the bf16 matrix cores at fp32 accuracy
// (three exact bf16 pieces per fp32 factor, see tq_bf3.h):
//     x~_i[k] = nu_i ( sum_j c[idx_ij] Pi[j][k]  +  kappa gamma_i sum_j z_ij S[j][k] ).
// The VECTOR is the row of the MFMA and the output coordinate the column, so
//   * the A operand (lane = vector, 8 consecutive j) is exactly what decoding 8 coordinates of one code
//     yields: a lane decodes its code's bit planes straight into the operand registers, no staging;
//   * the B operand is a piece of Pi^T / S^T (row k, 8 consecutive j), resident in LDS for the life of the
//     workgroup.  The three pieces of both matrices take 6 x 32 KB, so a workgroup holds the rows of HALF the
//     output coordinates (blockIdx.y) and every code is decoded by two workgroups;
//   * D[vector][k] is stored as 128 contiguous bytes per vector and half-wave.
// Workgroup = 8 wavefronts; a wavefront takes 32 vectors per round (all of k = 0..127 in 8 steps of 16, two
// 32-column sub-tiles), workgroups stride over the blocks of 256 vectors.
#include "tq_bf3.h"

namespace tq {

namespace {

constexpr int LDJ = 136;  // bf16 per LDS row: 128 values of j + 8 padding (272 bytes: conflict-free 16-byte reads)
constexpr int MAT_ELEMS = 3 * 64 * LDJ;

struct Dq128Args {
  const uint32_t* idx;
  const uint32_t* qjl;
  const float* gamma;
  const float* norm;  // nullable
  const float* PiT;
  const float* ST;
  float* out;
  int64_t ldo;
  int64_t n;
  float kappa;
  Codebook cb;
};

template <int BITS, bool PROD>
__global__ __launch_bounds__(512) void dequant128_bf3_kernel(const Dq128Args a) {
  constexpr int PC = BITS == 0 ? 0 : BITS == 1 ? 1 : 3;  // pieces of a decoded centroid (1 bit: +-c_1, c_1 applied at the end)
  constexpr int NB = BITS > 0 ? BITS : 1;
  constexpr int MATS = (BITS > 0 ? 1 : 0) + (PROD ? 1 : 0);
  extern __shared__ __attribute__((aligned(16))) unsigned short lds_s[];  // [matrix][piece][k 64][LDJ], then the table
  uint2* const table_s = reinterpret_cast<uint2*>(lds_s + MATS * MAT_ELEMS);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = blockIdx.y;  // output coordinates [64 half, 64 half + 64)

  // ---- the rows of Pi^T (and S^T) of this half, split into pieces ---------------------------------
  {
    int m = 0;
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      if (s == 0 ? BITS == 0 : !PROD) continue;
      const float* W = (s == 0 ? a.PiT : a.ST) + (int64_t)(64 * half) * 128;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int e = (i * 512 + tid) * 4;  // element of the 64 x 128 block
        const int k = e >> 7, j = e & 127;
        const f32x4 v = *reinterpret_cast<const f32x4*>(W + e);
        uint32_t lo[3], hi[3];
        split3_pair(f32x2{v[0], v[1]}, lo[0], lo[1], lo[2]);
        split3_pair(f32x2{v[2], v[3]}, hi[0], hi[1], hi[2]);
#pragma unroll
        for (int pc = 0; pc < 3; ++pc)
          *reinterpret_cast<uint2*>(lds_s + m * MAT_ELEMS + (pc * 64 + k) * LDJ + j) = make_uint2(lo[pc], hi[pc]);
      }
      ++m;
    }
    if (PC == 3 && tid < 16) {
      uint32_t p1, p2, p3;
      split3(a.cb.c[tid], p1, p2, p3);
      table_s[tid] = make_uint2(p1 | (p2 << 16), p3);
    }
  }
  __syncthreads();

  const int vi = lane & 31, jg = lane >> 5;  // A: vector within the round, which 8 of the 16 values of j
  const float c1 = BITS == 1 ? a.cb.c[1] : 1.f;
  const int64_t blocks = (a.n + 255) / 256;

  uint32_t w[4][NB], z[4], wn[4][NB], zn[4];
  float nu = 0.f, kg = 0.f, nun = 0.f, kgn = 0.f;
  auto load_code = [&](int64_t blk) {  // into the "next" registers
    const int64_t v = blk * 256 + wave * 32 + vi;
    const int64_t row = v < a.n ? v : a.n - 1;  // clamped: such rows are not stored
#pragma unroll
    for (int g = 0; g < 4; ++g) {
#pragma unroll
      for (int pl = 0; pl < BITS; ++pl) wn[g][pl] = a.idx[row * (4 * BITS) + g * BITS + pl];
      zn[g] = PROD ? a.qjl[row * 4 + g] : 0u;
    }
    nun = a.norm != nullptr ? a.norm[row] : 1.f;
    kgn = PROD ? a.kappa * a.gamma[row] : 0.f;
  };

  load_code(blockIdx.x);
  for (int64_t blk = blockIdx.x; blk < blocks; blk += gridDim.x) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
#pragma unroll
      for (int pl = 0; pl < BITS; ++pl) w[g][pl] = wn[g][pl];
      z[g] = zn[g];
    }
    nu = nun;
    kg = kgn;
    load_code(blk + gridDim.x);  // the next round's code travels during this round (clamped past the end)
    floatx16 acc1[2], acc2[2];
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        acc1[ct][r] = 0.f;
        acc2[ct][r] = 0.f;
      }
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const int g = s >> 1, off = (s & 1) * 16 + 8 * jg;  // word of the code, first bit
      const int j0 = 16 * s + 8 * jg;
      // ---- A operands: this lane's 8 coordinates decoded into pieces --------------------------------
      bf16x8 ca[PC > 0 ? PC : 1], za;
      if (PC == 1) {
        u32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          v[e] = 0xBF80BF80u ^ (((w[g][0] >> (off + 2 * e)) & 1u) << 15) ^ (((w[g][0] >> (off + 2 * e + 1)) & 1u) << 31);
        ca[0] = *reinterpret_cast<const bf16x8*>(&v);
      } else if (PC == 3) {
        uint32_t lv[2] = {0u, 0u};  // bucket numbers of 4 coordinates, one per byte
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int pl = 0; pl < BITS; ++pl)
            lv[h] |= ((((w[g][pl] >> (off + 4 * h)) & 0xFu) * 0x00204081u) & 0x01010101u) << pl;
        uint2 e[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) e[u] = table_s[(lv[u >> 2] >> (8 * (u & 3))) & 0xFFu];
        u32x4 v1, v2, v3;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          v1[u] = __builtin_amdgcn_perm(e[2 * u + 1].x, e[2 * u].x, 0x05040100u);
          v2[u] = __builtin_amdgcn_perm(e[2 * u + 1].x, e[2 * u].x, 0x07060302u);
          v3[u] = __builtin_amdgcn_perm(e[2 * u + 1].y, e[2 * u].y, 0x05040100u);
        }
        ca[0] = *reinterpret_cast<const bf16x8*>(&v1);
        ca[PC >= 3 ? 1 : 0] = *reinterpret_cast<const bf16x8*>(&v2);
        ca[PC >= 3 ? 2 : 0] = *reinterpret_cast<const bf16x8*>(&v3);
      }
      if (PROD) {
        u32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          v[e] = 0xBF80BF80u ^ (((z[g] >> (off + 2 * e)) & 1u) << 15) ^ (((z[g] >> (off + 2 * e + 1)) & 1u) << 31);
        za = *reinterpret_cast<const bf16x8*>(&v);
      }
      // ---- B operands from LDS, MFMAs -------------------------------------------------------------
#pragma unroll
      for (int ct = 0; ct < 2; ++ct) {
        const unsigned short* const brow = lds_s + (32 * ct + vi) * LDJ + j0;  // row k = 32 ct + lane % 32 of a piece
        int m = 0;
        if (BITS > 0) {
          bf16x8 pb[3];
#pragma unroll
          for (int pc = 0; pc < 3; ++pc) pb[pc] = *reinterpret_cast<const bf16x8*>(brow + m * MAT_ELEMS + pc * 64 * LDJ);
          if (PC == 1) {
#pragma unroll
            for (int pc = 2; pc >= 0; --pc) acc1[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ca[0], pb[pc], acc1[ct], 0, 0, 0);
          } else {
            constexpr int TA[6] = {2, 1, 0, 1, 0, 0};  // centroid piece; smallest products first
            constexpr int TB[6] = {0, 1, 2, 0, 1, 0};  // matrix piece
#pragma unroll
            for (int t = 0; t < 6; ++t)
              acc1[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ca[PC >= 3 ? TA[t] : 0], pb[TB[t]], acc1[ct], 0, 0, 0);
          }
          ++m;
        }
        if (PROD) {
#pragma unroll
          for (int pc = 2; pc >= 0; --pc) {
            const bf16x8 pb = *reinterpret_cast<const bf16x8*>(brow + m * MAT_ELEMS + pc * 64 * LDJ);
            acc2[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(za, pb, acc2[ct], 0, 0, 0);
          }
        }
      }
      // keep the steps apart: hoisting every step's operand reads to the top costs more registers than there are
      __builtin_amdgcn_sched_barrier(0);
    }
    // ---- epilogue: D[vector][k]; the factors of a row's vector sit in the lane with that number --------
    const int64_t v0 = blk * 256 + wave * 32;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = 8 * (r >> 2) + (r & 3) + 4 * (lane >> 5);
      const float rnu = __int_as_float(__builtin_amdgcn_ds_bpermute(4 * row, __float_as_int(nu)));
      const float rkg = __int_as_float(__builtin_amdgcn_ds_bpermute(4 * row, __float_as_int(kg)));
      if (v0 + row < a.n) {
        float* o = a.out + (v0 + row) * a.ldo + 64 * half + vi;
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) o[32 * ct] = rnu * fmaf(rkg, acc2[ct][r], c1 * acc1[ct][r]);
      }
    }
  }
}

template <int BITS, bool PROD>
hipError_t launch_one(const Dq128Args& a, hipStream_t s) {
  constexpr int MATS = (BITS > 0 ? 1 : 0) + (PROD ? 1 : 0);
  constexpr int lds = MATS * MAT_ELEMS * 2 + 16 * 8;
  static bool attr_done = false;  // per instantiation: the limit has to be raised once
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&dequant128_bf3_kernel<BITS, PROD>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  const int64_t blocks = (a.n + 255) / 256;
  const dim3 grid((unsigned)(blocks < 128 ? blocks : 128), 2);  // one workgroup per compute unit
  hipLaunchKernelGGL((dequant128_bf3_kernel<BITS, PROD>), grid, dim3(512), lds, s, a);
  return hipGetLastError();
}

}  // namespace

// d = 128, one instance; a 1-bit table must be +-c
bool dequant128_bf3_applicable(int bits, bool prod, const Codebook& cb) {
  if (bits < 0 || bits > 4 || (bits == 0 && !prod)) return false;
  return bits != 1 || cb.c[0] == -cb.c[1];
}

hipError_t launch_dequant128_bf3(int bits, bool prod, const uint32_t* idx, const uint32_t* qjl, const float* gamma,
                                 const float* norm, const float* PiT, const float* ST, float* out, int64_t ldo, int64_t n,
                                 float kappa, const Codebook& cb, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  Dq128Args a;
  a.idx = idx; a.qjl = qjl; a.gamma = gamma; a.norm = norm; a.PiT = PiT; a.ST = ST; a.out = out; a.ldo = ldo; a.n = n;
  a.kappa = kappa; a.cb = cb;
  switch (bits * 2 + (prod ? 1 : 0)) {
    case 1: return launch_one<0, true>(a, s);
    case 2: return launch_one<1, false>(a, s);
    case 3: return launch_one<1, true>(a, s);
    case 4: return launch_one<2, false>(a, s);
    case 5: return launch_one<2, true>(a, s);
    case 6: return launch_one<3, false>(a, s);
    case 7: return launch_one<3, true>(a, s);
    case 8: return launch_one<4, false>(a, s);
    case 9: return launch_one<4, true>(a, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace tq
