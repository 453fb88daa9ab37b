// Per-query top-k over a row of scores (the "return top-10" step of the ANN
// configurations).  One workgroup per row: every thread keeps its own sorted
// list of the k best (value, index) it has seen while striding over the row,
// then the 256 lists are merged by k rounds of a workgroup-wide arg-max.
// Order: larger score first; equal scores by lower index.
// A few long rows (one query against a million codes) would leave the chip to
// a few workgroups: such rows are cut into chunks, one workgroup per (row,
// chunk) writes the chunk's k best pairs, and launch_topk_merge joins them.
#include "tq_internal.h"

namespace tq {

__device__ __forceinline__ bool better(float va, int ia, float vb, int ib) {
  return va > vb || (va == vb && ia < ib);
}

template <int KMAX>
__global__ __launch_bounds__(256) void topk_kernel(const float* __restrict__ scores, const int64_t n_row,
                                                   const int64_t ld, const int k, const int vec4,
                                                   int32_t* __restrict__ out_idx,
                                                   float* __restrict__ out_val, const int64_t chunk_len) {
  extern __shared__ unsigned char smem_raw[];
  float* cand_v = reinterpret_cast<float*>(smem_raw);            // [256 * k]
  int* cand_i = reinterpret_cast<int*>(cand_v + 256 * k);        // [256 * k]
  __shared__ float red_v[4];
  __shared__ int red_i[4];
  __shared__ int red_slot[4];

  const int tid = threadIdx.x;
  // chunk_len > 0: workgroup (row, chunk) takes columns [c0, c0 + chunk_len) of the row (chunk_len is a multiple of
  // 4, so a chunk is as aligned as the row) and writes k (value, index) pairs, -inf / INT_MAX where it has fewer
  const int64_t c0 = chunk_len > 0 ? (int64_t)blockIdx.y * chunk_len : 0;
  const int64_t n = chunk_len > 0 ? (n_row - c0 < chunk_len ? n_row - c0 : chunk_len) : n_row;
  const float* row = scores + (int64_t)blockIdx.x * ld + c0;
  const int64_t out_row = chunk_len > 0 ? (int64_t)blockIdx.x * gridDim.y + blockIdx.y : blockIdx.x;
  const float NEG = -__builtin_inff();

  float bv[KMAX];
  int bi[KMAX];
#pragma unroll
  for (int j = 0; j < KMAX; ++j) {
    bv[j] = NEG;
    bi[j] = 0x7fffffff;
  }
  // position k-1 of a thread's list is its current worst kept entry: almost every element is
  // rejected by one compare against it
  float worst_v = NEG;
  int worst_i = 0x7fffffff;
  auto consider = [&](float v, int id) {
    if (better(v, id, worst_v, worst_i)) {
      // insert by a single pass of compare-exchange from the top
#pragma unroll
      for (int j = 0; j < KMAX; ++j) {
        if (j < k && better(v, id, bv[j], bi[j])) {
          const float tv = bv[j];
          const int ti = bi[j];
          bv[j] = v;
          bi[j] = id;
          v = tv;
          id = ti;
        }
        if (j == k - 1) {
          worst_v = bv[j];
          worst_i = bi[j];
        }
      }
    }
  };
  if (vec4) {
    // 16-byte loads, four of them in flight per thread before any compare
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const f32x4* row4 = reinterpret_cast<const f32x4*>(row);
    const int64_t n4 = n >> 2;
    constexpr int U = 4;
    for (int64_t i0 = tid; i0 < n4; i0 += 256 * U) {
      f32x4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int64_t i = i0 + 256 * u;
        v[u] = i < n4 ? __builtin_nontemporal_load(row4 + i) : f32x4{NEG, NEG, NEG, NEG};
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (i0 + 256 * u >= n4) break;  // padding of the last round: no element, no index
        const int id = (int)(c0 + ((i0 + 256 * u) << 2));
        consider(v[u].x, id);
        consider(v[u].y, id + 1);
        consider(v[u].z, id + 2);
        consider(v[u].w, id + 3);
      }
    }
    for (int64_t i = (n4 << 2) + tid; i < n; i += 256) consider(row[i], (int)(c0 + i));
  } else {
    for (int64_t i = tid; i < n; i += 256) consider(row[i], (int)(c0 + i));
  }
#pragma unroll
  for (int j = 0; j < KMAX; ++j)
    if (j < k) {
      cand_v[tid * k + j] = bv[j];
      cand_i[tid * k + j] = bi[j];
    }
  __syncthreads();

  // k rounds: each thread's list is sorted, so its best remaining entry is at
  // its own cursor; the workgroup picks the best of the 256 cursors.
  int cursor = 0;
  for (int r = 0; r < k; ++r) {
    float v = (cursor < k) ? cand_v[tid * k + cursor] : NEG;
    int id = (cursor < k) ? cand_i[tid * k + cursor] : 0x7fffffff;
    int who = tid;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const float ov = __shfl_xor(v, off);
      const int oi = __shfl_xor(id, off);
      const int ow = __shfl_xor(who, off);
      if (better(ov, oi, v, id)) {
        v = ov;
        id = oi;
        who = ow;
      }
    }
    if ((tid & 63) == 0) {
      red_v[tid >> 6] = v;
      red_i[tid >> 6] = id;
      red_slot[tid >> 6] = who;
    }
    __syncthreads();
    float fv = red_v[0];
    int fi = red_i[0], fw = red_slot[0];
#pragma unroll
    for (int w = 1; w < 4; ++w)
      if (better(red_v[w], red_i[w], fv, fi)) {
        fv = red_v[w];
        fi = red_i[w];
        fw = red_slot[w];
      }
    if (tid == fw) ++cursor;
    if (tid == 0) {
      out_idx[out_row * k + r] = (fi == 0x7fffffff && chunk_len == 0) ? -1 : fi;
      if (out_val != nullptr) out_val[out_row * k + r] = fv;
    }
    __syncthreads();
  }
}

// Chunks per row when a call's rows are too few to fill the chip: 0 (one workgroup per row) unless the rows are
// few and long; then chunks of at least 8192 scores, about four workgroups per compute unit in all, and no more
// pairs per row than the joining kernel takes (4096).  (Short chunks are the cheaper ones: while a thread has seen
// fewer than some hundred scores nearly every score enters some lane's list, so a wavefront pays the insertion
// for every element; one row of 10^6 scores: 35 us in 122 chunks, 103 us in 30.)
int topk_chunks(int64_t rows, int64_t n, int k) {
  if (k < 1 || rows < 1 || rows > 128 || n < 65536) return 0;
  int64_t c = (4 * (int64_t)device_cu_count() + rows - 1) / rows;
  if (c > n / 8192) c = n / 8192;
  if (c > 4096 / k) c = 4096 / k;
  if (c > 65535) c = 65535;
  return c >= 2 ? (int)c : 0;
}

// chunks == 0: the rows' k best straight to out_idx / out_val.  chunks > 0 (from topk_chunks): the k best of every
// chunk to part_idx / part_val [rows][chunks][k], to be joined by launch_topk_merge.
hipError_t launch_topk(const float* scores, int64_t rows, int64_t n, int64_t ld, int k,
                       int32_t* out_idx, float* out_val, hipStream_t stream, int chunks, float* part_val,
                       int32_t* part_idx) {
  if (rows == 0 || k == 0) return hipSuccess;
  if (k < 1 || k > 64 || rows > 0x7fffffff || n > 0x7fffffff) return hipErrorInvalidValue;
  if (chunks > 0 && (part_val == nullptr || part_idx == nullptr || chunks > 65535)) return hipErrorInvalidValue;
  const size_t smem = (size_t)256 * k * 8;
  const int vec4 = (ld % 4 == 0) && ((reinterpret_cast<uintptr_t>(scores) & 15u) == 0);
  const int64_t chunk_len = chunks > 0 ? ((n + chunks - 1) / chunks + 3) / 4 * 4 : 0;
  const dim3 grid((unsigned)rows, chunks > 0 ? (unsigned)chunks : 1u);
  if (chunks > 0) {
    out_idx = part_idx;
    out_val = part_val;
  }
  if (k <= 16)
    hipLaunchKernelGGL((topk_kernel<16>), grid, dim3(256), smem, stream, scores, n, ld, k, vec4, out_idx, out_val, chunk_len);
  else {
    // more than 64 KB of dynamic LDS has to be allowed explicitly
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&topk_kernel<64>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((topk_kernel<64>), grid, dim3(256), smem, stream, scores, n, ld, k, vec4, out_idx, out_val, chunk_len);
  }
  return hipGetLastError();
}

}  // namespace tq
