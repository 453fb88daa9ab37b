// Scoring when only a few queries share each code (decode attention with
// grouped queries: 4 query heads per KV head).  There is no operand reuse to
// speak of, so the kernel is organised around the stream of codes:
//
//   lane = key.  A wavefront takes 64 consecutive keys, each lane loads its own
//   key's packed words for 128 coordinates at a time (16-byte loads, fully
//   coalesced across the wave), expands them coordinate by coordinate in
//   registers and feeds v_mfma_f32_4x4x1_16b_f32:  16 independent 4x4 blocks,
//   A = 4 query values (one per lane of a block), B = 4 key values (one per
//   lane of a block), so one instruction multiplies one coordinate of 64 keys
//   by 4 queries.  Lane l = 4*block + j ends up with D[i][j] in register i =
//   the score of query i against its own key.
//
// The rotated / sketched queries (Pi q, S q) come from a small matrix-vector
// kernel and sit in LDS laid out [k/4][query][k%4], so one 16-byte read gives a
// lane the values of its query (lane%4) for four consecutive coordinates.
#include "tq_internal.h"

namespace tq {

typedef float floatx4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// out[q][j] = sum_k W[j][k] x[q][k] for a handful of queries.  One thread per
// output (q, j), j fastest; a workgroup stages its queries in LDS and every
// thread walks its own row of W with 16-byte loads (each 128-byte line of W is
// consumed by the thread that fetched it).  blockIdx.z selects (W0, out0) or
// (W1, out1); blockIdx.y a block of 4 queries; blockIdx.x a block of 64 rows j.
// ---------------------------------------------------------------------------
constexpr int MV_Q = 4;

__global__ __launch_bounds__(256) void matvec_small_kernel(const int d, const int nq,
                                                           const float* __restrict__ W0,
                                                           const float* __restrict__ W1,
                                                           const float* __restrict__ x, const int64_t ldx,
                                                           float* __restrict__ out0,
                                                           float* __restrict__ out1) {
  extern __shared__ __attribute__((aligned(16))) float xs[];  // [MV_Q][d]
  const int tid = threadIdx.x;
  const int q0 = blockIdx.y * MV_Q;
  for (int e = tid; e < MV_Q * d; e += 256) {
    const int r = e / d, k = e - r * d;
    xs[e] = (q0 + r < nq) ? x[(int64_t)(q0 + r) * ldx + k] : 0.f;
  }
  __syncthreads();
  const int j = blockIdx.x * 64 + (tid & 63);
  const int r = tid >> 6;  // query within the block of 4: one per wavefront
  if (j >= d || q0 + r >= nq) return;
  const float4* w4 = reinterpret_cast<const float4*>((blockIdx.z == 0 ? W0 : W1) + (int64_t)j * d);
  const float4* x4 = reinterpret_cast<const float4*>(xs + r * d);
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll 8
  for (int k4 = 0; k4 < d / 4; ++k4) {
    const float4 w = w4[k4];
    const float4 v = x4[k4];
    a0 = fmaf(w.x, v.x, a0);
    a1 = fmaf(w.y, v.y, a1);
    a2 = fmaf(w.z, v.z, a2);
    a3 = fmaf(w.w, v.w, a3);
  }
  (blockIdx.z == 0 ? out0 : out1)[(int64_t)(q0 + r) * d + j] = (a0 + a1) + (a2 + a3);
}

// The same product for long vectors: one wavefront per output row j, its lanes striding over the row with
// 16-byte loads (a wavefront's load is 1 KB of one row; a thread per row, as above, touches 64 rows per load and
// walks each of them alone: 43 us at d = 1536, 110 us for two matrices at d = 3072).  Four rows per workgroup, the
// block of 4 queries in LDS; blockIdx.x: rows, .y: query block, .z: matrix.
__global__ __launch_bounds__(256) void matvec_rows_kernel(const int d, const int nq, const float* __restrict__ W0,
                                                          const float* __restrict__ W1, const float* __restrict__ x,
                                                          const int64_t ldx, float* __restrict__ out0,
                                                          float* __restrict__ out1, const int x_bf16) {
  extern __shared__ __attribute__((aligned(16))) float xs[];  // [MV_Q][d]
  const int tid = threadIdx.x, lane = tid & 63;
  const int q0 = blockIdx.y * MV_Q;
  for (int e = tid; e < MV_Q * d; e += 256) {
    const int r = e / d, k = e - r * d;
    float v = 0.f;
    if (q0 + r < nq)
      v = x_bf16 ? __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(x)[(int64_t)(q0 + r) * ldx + k] << 16)
                 : x[(int64_t)(q0 + r) * ldx + k];
    xs[e] = v;
  }
  __syncthreads();
  const int j = blockIdx.x * 4 + (tid >> 6);
  if (j >= d) return;  // the whole wavefront
  const float4* w4 = reinterpret_cast<const float4*>((blockIdx.z == 0 ? W0 : W1) + (int64_t)j * d);
  float acc[MV_Q] = {0.f, 0.f, 0.f, 0.f};
  for (int k4 = lane; k4 < d / 4; k4 += 64) {
    const float4 w = w4[k4];
#pragma unroll
    for (int r = 0; r < MV_Q; ++r) {
      const float4 v = reinterpret_cast<const float4*>(xs + r * d)[k4];
      acc[r] = fmaf(w.x, v.x, fmaf(w.y, v.y, fmaf(w.z, v.z, fmaf(w.w, v.w, acc[r]))));
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1)
#pragma unroll
    for (int r = 0; r < MV_Q; ++r) acc[r] += __shfl_xor(acc[r], off);
  if (lane < MV_Q && q0 + lane < nq) {
    const float v = lane == 0 ? acc[0] : lane == 1 ? acc[1] : lane == 2 ? acc[2] : acc[3];
    (blockIdx.z == 0 ? out0 : out1)[(int64_t)(q0 + lane) * d + j] = v;
  }
}

// Alg. 1 for a handful of long vectors (adding to an index one vector at a time): y = Pi x by the row-per-wavefront
// kernel above, then one workgroup per vector takes the norm of x, scales, decides and packs.  (The tiled contraction
// walks d / 32 k-steps in series whatever the batch: 78 us for one vector at d = 1536.)  Rotating first and dividing
// by the norm afterwards differs from the other kernels' order by rounding only.
// ew != NULL (Alg. 2): the residual in the rotated basis, e = y - c[idx], goes to ew [n][d] and its norm to gamma.
template <int BITS>
__global__ __launch_bounds__(256) void quant_rows_finish_kernel(const int d, const void* __restrict__ x, const int64_t ldx,
                                                                const int x_bf16, const float* __restrict__ yw,
                                                                const Codebook cb, uint32_t* __restrict__ idx,
                                                                float* __restrict__ norm, float* __restrict__ ew,
                                                                float* __restrict__ gamma) {
  __shared__ float red_s[4];
  __shared__ float red_e[4];
  const int tid = threadIdx.x, lane = tid & 63;
  const int64_t row = blockIdx.x;
  float inv = 1.f;
  if (norm != nullptr) {
    float ss = 0.f;
    for (int k = tid; k < d; k += 256) {
      const float v = x_bf16 ? __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(x)[row * ldx + k] << 16)
                             : reinterpret_cast<const float*>(x)[row * ldx + k];
      ss = fmaf(v, v, ss);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
    if (lane == 0) red_s[tid >> 6] = ss;
    __syncthreads();
    const float nu = sqrtf((red_s[0] + red_s[1]) + (red_s[2] + red_s[3]));
    inv = nu > 0.f ? 1.f / nu : 0.f;  // a zero row stays zero
    if (tid == 0) norm[row] = nu;
  }
  if (BITS == 0 && ew == nullptr) return;
  const int groups = d >> 5;
  float ee = 0.f;
  for (int j0 = 0; j0 < d; j0 += 256) {  // uniform trip count; a wavefront covers 64 consecutive coordinates
    const int j = j0 + tid;
    int code = 0;
    if (j < d) {
      const float y = yw[row * d + j] * inv;
#pragma unroll
      for (int t = 0; t < (1 << BITS) - 1; ++t) code += (y >= cb.t[t]) ? 1 : 0;  // on a boundary: the upper cell
      if (ew != nullptr) {
        float c = cb.c[0];
#pragma unroll
        for (int t = 1; t < (1 << BITS); ++t) c = code == t ? cb.c[t] : c;
        const float e = y - c;
        ew[row * d + j] = e;
        ee = fmaf(e, e, ee);
      }
    }
    const int g = (j0 + (tid & ~63)) >> 5;  // first of the wavefront's two groups of 32
#pragma unroll
    for (int pl = 0; pl < BITS; ++pl) {
      const unsigned long long m = __ballot((code >> pl) & 1);
      if (lane == 0 && g < groups) idx[row * (int64_t)(groups * BITS) + g * BITS + pl] = (uint32_t)m;
      if (lane == 32 && g + 1 < groups) idx[row * (int64_t)(groups * BITS) + (g + 1) * BITS + pl] = (uint32_t)(m >> 32);
    }
  }
  if (ew != nullptr) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) ee += __shfl_xor(ee, off);
    if (lane == 0) red_e[tid >> 6] = ee;
    __syncthreads();
    if (tid == 0) gamma[row] = sqrtf((red_e[0] + red_e[1]) + (red_e[2] + red_e[3]));
  }
}

hipError_t launch_quant_rows(int bits, bool bf16, const void* x, int64_t ldx, int64_t n, int d, const float* Pi,
                             const Codebook& cb, float* yw, uint32_t* idx, float* norm, hipStream_t stream,
                             const float* SPiT, float* ew, uint32_t* qjl, float* gamma) {
  if (n == 0) return hipSuccess;
  if (n > 65535 * MV_Q || d % 32 != 0 || (size_t)MV_Q * d * sizeof(float) > 65536) return hipErrorInvalidValue;
  hipLaunchKernelGGL(matvec_rows_kernel, dim3((d + 3) / 4, (unsigned)((n + MV_Q - 1) / MV_Q), 1), dim3(256),
                     (size_t)MV_Q * d * sizeof(float), stream, d, (int)n, Pi, nullptr, static_cast<const float*>(x), ldx, yw,
                     nullptr, bf16 ? 1 : 0);
  if (const hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  const dim3 grid((unsigned)n);
  const int xb = bf16 ? 1 : 0;
  switch (bits) {
    case 0: hipLaunchKernelGGL(quant_rows_finish_kernel<0>, grid, dim3(256), 0, stream, d, x, ldx, xb, yw, cb, idx, norm, ew, gamma); break;
    case 1: hipLaunchKernelGGL(quant_rows_finish_kernel<1>, grid, dim3(256), 0, stream, d, x, ldx, xb, yw, cb, idx, norm, ew, gamma); break;
    case 2: hipLaunchKernelGGL(quant_rows_finish_kernel<2>, grid, dim3(256), 0, stream, d, x, ldx, xb, yw, cb, idx, norm, ew, gamma); break;
    case 3: hipLaunchKernelGGL(quant_rows_finish_kernel<3>, grid, dim3(256), 0, stream, d, x, ldx, xb, yw, cb, idx, norm, ew, gamma); break;
    case 4: hipLaunchKernelGGL(quant_rows_finish_kernel<4>, grid, dim3(256), 0, stream, d, x, ldx, xb, yw, cb, idx, norm, ew, gamma); break;
    default: return hipErrorInvalidValue;
  }
  if (const hipError_t e = hipGetLastError(); e != hipSuccess || ew == nullptr) return e;
  // Alg. 2: u = (S Pi^T) e, again one wavefront per matrix row (into the buffer the rotation has left), signs packed
  hipLaunchKernelGGL(matvec_rows_kernel, dim3((d + 3) / 4, (unsigned)((n + MV_Q - 1) / MV_Q), 1), dim3(256),
                     (size_t)MV_Q * d * sizeof(float), stream, d, (int)n, SPiT, nullptr, ew, (int64_t)d, yw, nullptr, 0);
  if (const hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  return launch_stage_sign_pack(d, yw, n, qjl, stream);
}

// DeQuant of Alg. 1 / Alg. 2 for a handful of long vectors: x~[k] = nu (sum_j Pi^T[k][j] c[idx_j] + kappa gamma
// sum_j S^T[k][j] z_j), one wavefront per output coordinate k (a row of Pi^T and of S^T, 1 KB per load), the decoded
// codes of Q vectors in LDS (4 for Alg. 1; 2 for Alg. 2, whose sign vector sits beside them).
template <int BITS, bool PROD>
__global__ __launch_bounds__(256) void dequant_rows_kernel(const int d, const int n, const uint32_t* __restrict__ idx,
                                                           const uint32_t* __restrict__ qjl, const float* __restrict__ gamma,
                                                           const float* __restrict__ norm, const float* __restrict__ PiT,
                                                           const float* __restrict__ ST, const Codebook cb, const float kappa,
                                                           float* __restrict__ out, const int64_t ldo) {
  constexpr int Q = PROD ? 2 : 4;
  extern __shared__ __attribute__((aligned(16))) float ys[];  // [Q][d], then (PROD) [Q][d] of +-kappa gamma
  __shared__ float cent_s[16];
  float* const zs = ys + Q * d;
  const int tid = threadIdx.x, lane = tid & 63;
  const int q0 = blockIdx.y * Q;
  if (tid < 16) cent_s[tid] = cb.c[tid];
  __syncthreads();
  const int groups = d >> 5;
  for (int e = tid; e < Q * d; e += 256) {
    const int r = e / d, k = e - r * d;
    const int64_t row = q0 + r;
    float y = 0.f, z = 0.f;
    if (row < n) {
      int code = 0;
#pragma unroll
      for (int pl = 0; pl < BITS; ++pl) code |= (int)((idx[row * (int64_t)(groups * BITS) + (k >> 5) * BITS + pl] >> (k & 31)) & 1u) << pl;
      y = cent_s[code];
      if (PROD) {
        const float kg = kappa * gamma[row];
        z = ((qjl[row * groups + (k >> 5)] >> (k & 31)) & 1u) ? kg : -kg;
      }
    }
    ys[e] = y;
    if (PROD) zs[e] = z;
  }
  __syncthreads();
  const int j = blockIdx.x * 4 + (tid >> 6);
  if (j >= d) return;  // the whole wavefront
  const float4* w4 = reinterpret_cast<const float4*>(PiT + (int64_t)j * d);
  const float4* s4 = PROD ? reinterpret_cast<const float4*>(ST + (int64_t)j * d) : nullptr;
  float acc[Q];
#pragma unroll
  for (int r = 0; r < Q; ++r) acc[r] = 0.f;
  for (int k4 = lane; k4 < d / 4; k4 += 64) {
    const float4 w = w4[k4];
    float4 sv = make_float4(0.f, 0.f, 0.f, 0.f);
    if (PROD) sv = s4[k4];
#pragma unroll
    for (int r = 0; r < Q; ++r) {
      const float4 v = reinterpret_cast<const float4*>(ys + r * d)[k4];
      acc[r] = fmaf(w.x, v.x, fmaf(w.y, v.y, fmaf(w.z, v.z, fmaf(w.w, v.w, acc[r]))));
      if (PROD) {
        const float4 u = reinterpret_cast<const float4*>(zs + r * d)[k4];
        acc[r] = fmaf(sv.x, u.x, fmaf(sv.y, u.y, fmaf(sv.z, u.z, fmaf(sv.w, u.w, acc[r]))));
      }
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1)
#pragma unroll
    for (int r = 0; r < Q; ++r) acc[r] += __shfl_xor(acc[r], off);
  if (lane < Q && q0 + lane < n) {
    float v = acc[0];
#pragma unroll
    for (int r = 1; r < Q; ++r) v = lane == r ? acc[r] : v;
    const float nu = norm != nullptr ? norm[q0 + lane] : 1.f;
    out[(int64_t)(q0 + lane) * ldo + j] = nu * v;
  }
}

template <int BITS>
static hipError_t dequant_rows_bits(bool prod, int d, int n, const uint32_t* idx, const uint32_t* qjl, const float* gamma,
                                    const float* norm, const float* PiT, const float* ST, const Codebook& cb, float kappa,
                                    float* out, int64_t ldo, hipStream_t s) {
  const int Q = prod ? 2 : 4;
  const dim3 grid((d + 3) / 4, (n + Q - 1) / Q);
  const size_t lds = (size_t)(prod ? 2 : 1) * Q * d * sizeof(float);
  if (prod)
    hipLaunchKernelGGL((dequant_rows_kernel<BITS, true>), grid, dim3(256), lds, s, d, n, idx, qjl, gamma, norm, PiT, ST, cb, kappa, out, ldo);
  else
    hipLaunchKernelGGL((dequant_rows_kernel<BITS, false>), grid, dim3(256), lds, s, d, n, idx, qjl, gamma, norm, PiT, ST, cb, kappa, out, ldo);
  return hipGetLastError();
}

hipError_t launch_dequant_rows(int bits, bool prod, int d, int64_t n, const uint32_t* idx, const uint32_t* qjl,
                               const float* gamma, const float* norm, const float* PiT, const float* ST, const Codebook& cb,
                               float kappa, float* out, int64_t ldo, hipStream_t s) {
  if (n == 0) return hipSuccess;
  if (n > 65535 || d % 32 != 0 || (size_t)4 * d * sizeof(float) > 65536) return hipErrorInvalidValue;
  switch (bits) {
    case 0: return dequant_rows_bits<0>(prod, d, (int)n, idx, qjl, gamma, norm, PiT, ST, cb, kappa, out, ldo, s);
    case 1: return dequant_rows_bits<1>(prod, d, (int)n, idx, qjl, gamma, norm, PiT, ST, cb, kappa, out, ldo, s);
    case 2: return dequant_rows_bits<2>(prod, d, (int)n, idx, qjl, gamma, norm, PiT, ST, cb, kappa, out, ldo, s);
    case 3: return dequant_rows_bits<3>(prod, d, (int)n, idx, qjl, gamma, norm, PiT, ST, cb, kappa, out, ldo, s);
    case 4: return dequant_rows_bits<4>(prod, d, (int)n, idx, qjl, gamma, norm, PiT, ST, cb, kappa, out, ldo, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_matvec_small(int d, int nq, const float* W0, const float* W1, const float* x,
                               int64_t ldx, float* out0, float* out1, hipStream_t stream) {
  if (nq == 0) return hipSuccess;
  if (d % 4 != 0 || (size_t)MV_Q * d * sizeof(float) > 65536) return hipErrorInvalidValue;
  if (d >= 512) {
    hipLaunchKernelGGL(matvec_rows_kernel, dim3((d + 3) / 4, (nq + MV_Q - 1) / MV_Q, W1 != nullptr ? 2 : 1), dim3(256),
                       (size_t)MV_Q * d * sizeof(float), stream, d, nq, W0, W1, x, ldx, out0, out1, 0);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(matvec_small_kernel, dim3((d + 63) / 64, (nq + MV_Q - 1) / MV_Q, W1 != nullptr ? 2 : 1),
                     dim3(256), (size_t)MV_Q * d * sizeof(float), stream, d, nq, W0, W1, x, ldx, out0, out1);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
struct ScoreSmallArgs {
  const float* qr;  // [n_groups*q_per_group][d]  Pi q
  const float* qs;  // [n_groups*q_per_group][d]  S q   (prod only)
  const uint32_t* idx;
  const uint32_t* qjl;
  const float* gamma;
  const float* norm;  // nullable
  float* scores;
  int64_t lds;
  int64_t n;          // keys per group
  int d;
  int q_per_group;
  float kappa;
  Codebook cb;
};

template <int BITS, bool PROD, int KPL>
__global__ __launch_bounds__(256) void score_small_kernel(const ScoreSmallArgs a) {
  extern __shared__ __attribute__((aligned(16))) float q_s[];  // qr then qs, each d*4 floats
  __shared__ float cent_s[16];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int group = blockIdx.y;
  const int pass = blockIdx.z;           // queries 4*pass .. 4*pass+3 of the group
  const int d = a.d;
  const int q0 = pass * 4;
  const int nq_here = min(4, a.q_per_group - q0);

  if (tid < 16) cent_s[tid] = a.cb.c[tid];
  // stage the queries: element (row r, coordinate k) -> [(k/4)*4 + r]*4 + k%4
  for (int e = tid; e < 4 * d; e += 256) {
    const int r = e / d, k = e - r * d;
    const int64_t qrow = (int64_t)group * a.q_per_group + q0 + r;
    const int dst = (((k >> 2) * 4 + r) << 2) + (k & 3);
    q_s[dst] = (r < nq_here) ? a.qr[qrow * d + k] : 0.f;
    if (PROD) q_s[4 * d + dst] = (r < nq_here) ? a.qs[qrow * d + k] : 0.f;
  }
  __syncthreads();

  const int words_per_row = (d / 32) * BITS;
  const int qw_per_row = d / 32;
  const int64_t gbase = (int64_t)group * a.n;
  const float4* qr4 = reinterpret_cast<const float4*>(q_s);
  const float4* qs4 = reinterpret_cast<const float4*>(q_s + 4 * d);

  // a wavefront owns 64*KPL consecutive keys; lane l takes keys base + u*64 + l.
  // The KPL keys of a lane share every query read and give independent MFMA chains.
  const int64_t base = ((int64_t)blockIdx.x * 4 + wave) * (64 * KPL);
  if (base >= a.n) return;
  int64_t row[KPL];
  bool valid[KPL];
  floatx4 acc[KPL], acc2[KPL];
#pragma unroll
  for (int u = 0; u < KPL; ++u) {
    const int64_t key = base + u * 64 + lane;
    valid[u] = key < a.n;
    row[u] = gbase + (valid[u] ? key : 0);
#pragma unroll
    for (int r = 0; r < 4; ++r) { acc[u][r] = 0.f; acc2[u][r] = 0.f; }
  }
  for (int c = 0; c < d / 128; ++c) {  // 128 coordinates = 4 groups of 32 at a time
    uint32_t w[KPL][4 * (BITS > 0 ? BITS : 1)];
    uint32_t zn[KPL][4];
#pragma unroll
    for (int u = 0; u < KPL; ++u) {
      if (BITS > 0) {
        const uint32_t* src = a.idx + row[u] * words_per_row + c * 4 * BITS;
#pragma unroll
        for (int v = 0; v < BITS; ++v) {  // 4*BITS words = BITS 16-byte loads
          const uint4 t = *reinterpret_cast<const uint4*>(src + 4 * v);
          w[u][4 * v] = t.x; w[u][4 * v + 1] = t.y; w[u][4 * v + 2] = t.z; w[u][4 * v + 3] = t.w;
        }
      }
      if (PROD) {
        const uint4 t = *reinterpret_cast<const uint4*>(a.qjl + row[u] * qw_per_row + c * 4);
        zn[u][0] = ~t.x; zn[u][1] = ~t.y; zn[u][2] = ~t.z; zn[u][3] = ~t.w;  // bit set = minus sign
      }
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
#pragma unroll
      for (int j4 = 0; j4 < 8; ++j4) {
        const float4 qa = qr4[((c * 32 + g * 8 + j4) << 2) + (lane & 3)];
        float4 qb = make_float4(0.f, 0.f, 0.f, 0.f);
        if (PROD) qb = qs4[((c * 32 + g * 8 + j4) << 2) + (lane & 3)];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int j = j4 * 4 + jj;
          const float av = jj == 0 ? qa.x : jj == 1 ? qa.y : jj == 2 ? qa.z : qa.w;
          const float bv = jj == 0 ? qb.x : jj == 1 ? qb.y : jj == 2 ? qb.z : qb.w;
#pragma unroll
          for (int u = 0; u < KPL; ++u) {
            if (BITS > 0) {
              uint32_t code = 0;
#pragma unroll
              for (int pl = 0; pl < BITS; ++pl) code |= ((w[u][g * BITS + pl] >> j) & 1u) << pl;
              acc[u] = __builtin_amdgcn_mfma_f32_4x4x1f32(av, cent_s[code], acc[u], 0, 0, 0);
            }
            if (PROD) {
              // +-1.0f with the sign bit taken from bit j of the inverted word
              const uint32_t sb = zn[u][g] << (31 - j);
              const float val = __uint_as_float((sb & 0x80000000u) | 0x3f800000u);
              acc2[u] = __builtin_amdgcn_mfma_f32_4x4x1f32(bv, val, acc2[u], 0, 0, 0);
            }
          }
        }
      }
    }
  }
#pragma unroll
  for (int u = 0; u < KPL; ++u) {
    if (valid[u]) {
      const float nu = a.norm != nullptr ? a.norm[row[u]] : 1.f;
      const float kg = PROD ? a.kappa * a.gamma[row[u]] : 0.f;
      const int64_t key = base + u * 64 + lane;
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (r < nq_here)
          a.scores[((int64_t)group * a.q_per_group + q0 + r) * a.lds + key] = nu * (acc[u][r] + kg * acc2[u][r]);
    }
  }
}

template <int BITS, bool PROD>
static hipError_t launch_kpl(const ScoreSmallArgs& a, int n_groups, size_t smem, hipStream_t s) {
  // two keys per lane once there is enough work to keep every SIMD busy anyway
  const bool big = a.n * (int64_t)n_groups >= (int64_t)1 << 19;
  const int kpl = big ? 2 : 1;
  const dim3 grid((unsigned)((a.n + 256 * kpl - 1) / (256 * kpl)), n_groups, (a.q_per_group + 3) / 4);
  if (big)
    hipLaunchKernelGGL((score_small_kernel<BITS, PROD, 2>), grid, dim3(256), smem, s, a);
  else
    hipLaunchKernelGGL((score_small_kernel<BITS, PROD, 1>), grid, dim3(256), smem, s, a);
  return hipGetLastError();
}

template <int BITS>
static hipError_t launch_bits(const ScoreSmallArgs& a, bool prod, int n_groups, size_t smem, hipStream_t s) {
  return prod ? launch_kpl<BITS, true>(a, n_groups, smem, s) : launch_kpl<BITS, false>(a, n_groups, smem, s);
}

hipError_t launch_score_small(int bits, bool prod, const float* qr, const float* qs, const uint32_t* idx,
                              const uint32_t* qjl, const float* gamma, const float* norm, float* scores,
                              int64_t lds, int64_t n, int d, int n_groups, int q_per_group, float kappa,
                              const Codebook& cb, hipStream_t stream) {
  if (n == 0 || n_groups == 0 || q_per_group == 0) return hipSuccess;
  if (d % 128 != 0 || d > 1024) return hipErrorInvalidValue;
  ScoreSmallArgs a;
  a.qr = qr; a.qs = qs; a.idx = idx; a.qjl = qjl; a.gamma = gamma; a.norm = norm;
  a.scores = scores; a.lds = lds; a.n = n; a.d = d; a.q_per_group = q_per_group;
  a.kappa = kappa; a.cb = cb;
  const size_t smem = (size_t)(prod ? 2 : 1) * 4 * d * sizeof(float);  // <= 32 KB
  switch (bits) {
    case 0: return launch_bits<0>(a, prod, n_groups, smem, stream);
    case 1: return launch_bits<1>(a, prod, n_groups, smem, stream);
    case 2: return launch_bits<2>(a, prod, n_groups, smem, stream);
    case 3: return launch_bits<3>(a, prod, n_groups, smem, stream);
    case 4: return launch_bits<4>(a, prod, n_groups, smem, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace tq
