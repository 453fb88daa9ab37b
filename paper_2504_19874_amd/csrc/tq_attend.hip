// Attention read-out over a quantised key/value cache (Sec. 4.3: the cache of past tokens is kept
// as codes).  For a query q of group g with logits_i = scale * score(q, key code i),
//     out = sum_i softmax(logits)_i * DeQuant(value code i).
// DeQuant is linear in the decoded code (Alg. 1: x~ = nu Pi^T c[idx]; Alg. 2 adds
// kappa gamma nu S^T z), so the weighted sum is taken over the DECODED CODES in the rotated
// basis and rotated back once per query:
//     out = Pi^T ( sum_i p_i nu_i c[idx_i] )  +  kappa S^T ( sum_i p_i nu_i gamma_i z_i ).
// The keys are split into chunks, one workgroup each (attend_values_kernel): it takes the chunk's
// maximum logit m, l = sum exp(logit - m) and the two rotated-basis sums with weights
// exp(logit - m); attend_combine_kernel joins the chunks of a query (weights exp(m_chunk - M) / L)
// and applies Pi^T and S^T.
//
// This file holds the kernels for any d (lane = coordinate, one key at a time); the d = 128
// kernel on the integer matrix cores is in tq_attend_128.hip.
#include "tq_attend.h"

namespace tq {

namespace {

constexpr int SIMPLE_CHUNK = 1024;

__device__ __forceinline__ float block_reduce(float v, bool take_max, float* red_s, int tid) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float u = __shfl_xor(v, o);
    v = take_max ? fmaxf(v, u) : v + u;
  }
  __syncthreads();  // red_s may still be read from the previous reduction
  if ((tid & 63) == 0) red_s[tid >> 6] = v;
  __syncthreads();
  v = red_s[0];
  for (int w = 1; w < (int)(blockDim.x >> 6); ++w) v = take_max ? fmaxf(v, red_s[w]) : v + red_s[w];
  return v;
}

template <bool PROD>
__global__ __launch_bounds__(256) void attend_values_kernel(const AttendArgs a) {
  __shared__ float w_s[4][SIMPLE_CHUNK];                                // exp(logit - m) * nu
  __shared__ float wg_s[PROD ? 4 : 1][PROD ? SIMPLE_CHUNK : 1];         // ... * gamma
  __shared__ float red_s[4];
  __shared__ float cent_s[16];
  const int tid = threadIdx.x;
  const int chunk = blockIdx.x, group = blockIdx.y, q0 = blockIdx.z * 4;
  const int64_t key0 = (int64_t)chunk * SIMPLE_CHUNK;
  const int nk = (int)(a.n - key0 < SIMPLE_CHUNK ? a.n - key0 : SIMPLE_CHUNK);
  const int64_t row0 = (int64_t)group * a.group_stride + key0;
  if (tid < 16) cent_s[tid] = a.cb.c[tid];

  float m[4], l[4];
#pragma unroll
  for (int qi = 0; qi < 4; ++qi) {
    const bool live = q0 + qi < a.q_per_group;
    const float* srow = a.scores + ((int64_t)group * a.q_per_group + q0 + (live ? qi : 0)) * a.lds + key0;
    float mx = -INFINITY;
    for (int k = tid; k < nk; k += 256) mx = fmaxf(mx, a.scale * srow[k]);
    m[qi] = block_reduce(mx, true, red_s, tid);
    float sum = 0.f;
    for (int k = tid; k < nk; k += 256) {
      const float w = expf(a.scale * srow[k] - m[qi]);
      sum += w;
      const float wn = w * a.norm[row0 + k];
      w_s[qi][k] = wn;
      if (PROD) wg_s[qi][k] = wn * a.gamma[row0 + k];
    }
    l[qi] = block_reduce(sum, false, red_s, tid);
  }
  __syncthreads();

  const int wpr = a.d / 32 * a.cb.bits, zpr = a.d / 32;
  const int64_t prow = ((int64_t)group * a.q_per_group + q0) * a.nchunks + chunk;  // + qi * nchunks
  for (int j = tid; j < a.d; j += 256) {
    const int g = j >> 5, bit = j & 31;
    float acc[4] = {0.f, 0.f, 0.f, 0.f}, accz[4] = {0.f, 0.f, 0.f, 0.f};
    for (int k = 0; k < nk; ++k) {
      const uint32_t* words = a.idx + (row0 + k) * wpr + g * a.cb.bits;
      int level = 0;
      for (int p = 0; p < a.cb.bits; ++p) level |= (int)((words[p] >> bit) & 1u) << p;
      const float c = cent_s[level];
      float z = 0.f;
      if (PROD) z = ((a.qjl[(row0 + k) * zpr + g] >> bit) & 1u) ? 1.f : -1.f;
#pragma unroll
      for (int qi = 0; qi < 4; ++qi) {
        acc[qi] = fmaf(w_s[qi][k], c, acc[qi]);
        if (PROD) accz[qi] = fmaf(wg_s[qi][k], z, accz[qi]);
      }
    }
#pragma unroll
    for (int qi = 0; qi < 4; ++qi) {
      if (q0 + qi >= a.q_per_group) continue;
      float* o = a.part + (prow + (int64_t)qi * a.nchunks) * attend_part_stride(a.d);
      o[4 + j] = acc[qi];
      o[4 + a.d + j] = accz[qi];
    }
  }
  if (tid < 4 && q0 + tid < a.q_per_group) {
    float* o = a.part + (prow + (int64_t)tid * a.nchunks) * attend_part_stride(a.d);
    o[0] = m[tid];
    o[1] = l[tid];
  }
}

// sum_j W[j * ld] * y[j] over j in [j0, j0 + count), 32 loads in flight
__device__ __forceinline__ float strided_dot(const float* W, int64_t ld, const float* y, int j0, int count) {
  float acc = 0.f;
  int j = j0;
  for (; j + 32 <= j0 + count; j += 32) {
    float v[32];
#pragma unroll
    for (int u = 0; u < 32; ++u) v[u] = W[(int64_t)(j + u) * ld];
#pragma unroll
    for (int u = 0; u < 32; ++u) acc = fmaf(v[u], y[j + u], acc);
  }
  for (; j < j0 + count; ++j) acc = fmaf(W[(int64_t)j * ld], y[j], acc);
  return acc;
}

// one workgroup per query: join the chunks, then back to the original basis
__global__ __launch_bounds__(256) void attend_combine_kernel(const float* part, int nchunks, int d, const float* Pi,
                                                             const float* S, float kappa, float* out, int64_t ldo) {
  extern __shared__ float sm[];  // y_s[2 d]: the two rotated-basis sums, normalised; e_s[nchunks]; o_s[256]
  __shared__ float red_s[4];
  float* const y_s = sm;
  float* const e_s = sm + 2 * d;
  float* const o_s = e_s + nchunks;
  const int tid = threadIdx.x;
  const int stride = attend_part_stride(d);
  const float* p = part + (int64_t)blockIdx.x * nchunks * stride;
  const int jmax = S != nullptr ? 2 * d : d;
  // d = 128: this thread's 64 + 64 matrix entries of the last step (thread = coordinate k and half of the j range)
  // are asked for before the chunks are joined, so the call has two dependent round trips to memory, not six
  const bool early = d == 128;
  float wp[64], ws[64];
  if (early) {
    const float* Pk = Pi + (tid >> 7) * 64 * 128 + (tid & 127);
#pragma unroll
    for (int u = 0; u < 64; ++u) wp[u] = Pk[u * 128];
    if (S != nullptr) {
      const float* Sk = S + (tid >> 7) * 64 * 128 + (tid & 127);
#pragma unroll
      for (int u = 0; u < 64; ++u) ws[u] = Sk[u * 128];
    }
  }
  if (nchunks == 0) {
    for (int j = tid; j < jmax; j += 256) y_s[j] = 0.f;  // no keys at all: the output is zero
  } else if (nchunks <= 32) {
    // the common case: every load of the joining step is issued at once (the chunk maxima and sums through
    // scalar registers), and every thread derives M and L for itself
    for (int j0 = 0; j0 < jmax; j0 += 256) {
      const int j = j0 + tid, jc = j < jmax ? j : jmax - 1;
      float v[32], mc[32], lc[32];
#pragma unroll
      for (int u = 0; u < 32; ++u) {  // unconditional loads (clamped), selected afterwards
        const int64_t base = (int64_t)(u < nchunks ? u : nchunks - 1) * stride;
        v[u] = p[base + 4 + jc];
        mc[u] = p[base];
        lc[u] = p[base + 1];
      }
#pragma unroll
      for (int u = 0; u < 32; ++u)
        if (u >= nchunks) mc[u] = -INFINITY;
      float M = mc[0];
#pragma unroll
      for (int u = 1; u < 32; ++u) M = fmaxf(M, mc[u]);
      float L = 0.f, acc = 0.f;
#pragma unroll
      for (int u = 0; u < 32; ++u) {
        const float e = expf(mc[u] - M);  // 0 past the last chunk
        L = fmaf(e, lc[u], L);
        acc = fmaf(e, v[u], acc);
      }
      if (j < jmax) y_s[j] = acc / L;
    }
  } else {
    // thread c holds (m, l) of chunk c, c + 256, ...
    float mx = -INFINITY;
    for (int c = tid; c < nchunks; c += 256) mx = fmaxf(mx, p[(int64_t)c * stride]);
    const float M = block_reduce(mx, true, red_s, tid);
    float ls = 0.f;
    for (int c = tid; c < nchunks; c += 256) {
      const float e = expf(p[(int64_t)c * stride] - M);
      e_s[c] = e;
      ls = fmaf(e, p[(int64_t)c * stride + 1], ls);
    }
    const float L = block_reduce(ls, false, red_s, tid);  // its barriers also publish e_s
    const float invL = L > 0.f ? 1.f / L : 0.f;
    for (int j = tid; j < jmax; j += 256) {
      float acc = 0.f;
      int c = 0;
      for (; c + 32 <= nchunks; c += 32) {  // 32 loads in flight
        float v[32];
#pragma unroll
        for (int u = 0; u < 32; ++u) v[u] = p[(int64_t)(c + u) * stride + 4 + j];
#pragma unroll
        for (int u = 0; u < 32; ++u) acc = fmaf(e_s[c + u], v[u], acc);
      }
      for (; c < nchunks; ++c) acc = fmaf(e_s[c], p[(int64_t)c * stride + 4 + j], acc);
      y_s[j] = acc * invL;
    }
  }
  __syncthreads();
  // out[k] = sum_j Pi[j][k] y[j] + kappa sum_j S[j][k] z[j]; for small d the j range is split over the threads
  const int parts = d <= 256 ? 256 / d : 1;
  const int span = d / parts;
  for (int k0 = 0; k0 < d; k0 += 256) {  // one trip unless d > 256
    const int item = k0 + tid, k = parts > 1 ? tid % d : item, part_ = parts > 1 ? tid / d : 0;
    float o = 0.f, oz = 0.f;
    if (early) {
      const int j0 = part_ * span;  // 64 * (tid / 128)
#pragma unroll
      for (int u = 0; u < 64; ++u) o = fmaf(wp[u], y_s[j0 + u], o);
      if (S != nullptr) {
#pragma unroll
        for (int u = 0; u < 64; ++u) oz = fmaf(ws[u], y_s[d + j0 + u], oz);
      }
    } else if (k < d && part_ < parts) {
      const int j0 = part_ * span;
      o = strided_dot(Pi + k, d, y_s, j0, span);
      if (S != nullptr) oz = strided_dot(S + k, d, y_s + d, j0, span);
    }
    o = fmaf(kappa, oz, o);
    if (parts > 1) {
      o_s[tid] = o;
      __syncthreads();
      if (tid < d) {
        for (int t = 1; t < parts; ++t) o += o_s[tid + t * d];
        out[(int64_t)blockIdx.x * ldo + tid] = o;
      }
    } else if (k < d) {
      out[(int64_t)blockIdx.x * ldo + k] = o;
    }
  }
}

}  // namespace

int attend_simple_chunks(int64_t n) { return (int)((n + SIMPLE_CHUNK - 1) / SIMPLE_CHUNK); }

hipError_t launch_attend_values(bool prod, const AttendArgs& a, int n_groups, hipStream_t s) {
  if (a.nchunks == 0 || n_groups == 0 || a.q_per_group == 0) return hipSuccess;
  const dim3 grid(a.nchunks, n_groups, (a.q_per_group + 3) / 4);
  if (prod)
    hipLaunchKernelGGL(attend_values_kernel<true>, grid, dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL(attend_values_kernel<false>, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_attend_combine(const float* part, int nchunks, int d, int64_t nq, const float* Pi, const float* S,
                                 float kappa, float* out, int64_t ldo, hipStream_t s) {
  if (nq == 0) return hipSuccess;
  hipLaunchKernelGGL(attend_combine_kernel, dim3((unsigned)nq), dim3(256), (2 * d + nchunks + 256) * sizeof(float), s, part, nchunks, d,
                     Pi, S, kappa, out, ldo);
  return hipGetLastError();
}

}  // namespace tq
