// HBM-bound codec stages: rotated coordinates -> packed indices, sketch values
// -> packed signs, packed indices -> centroid values; plus a square transpose
// used when deriving parameters.
//
// Packing uses the fact that a vector compare on a 64-wide wavefront IS a
// 64-bit ballot: with one coordinate per lane, "y >= t_k" for all 64 lanes
// lands in a scalar register pair, i.e. two finished 32-coordinate words.
// For ascending boundaries the masks are nested, and bit p of the bucket
// number (= how many boundaries are <= y) is the XOR of the masks whose
// position k satisfies k mod 2^p == 2^p - 1 (parity of floor(count / 2^p)).  So a b-bit decision costs
// 2^b - 1 compares per 64 coordinates and no per-lane integer work.
#include "tq_internal.h"

namespace tq {

constexpr int CHUNKS = 8;  // 64-coordinate chunks per wavefront iteration

template <int BITS, bool SIGN_ONLY>
__global__ __launch_bounds__(256) void stage_pack_kernel(const Codebook cb, const float* __restrict__ y,
                                                         const int64_t n_groups32,  // groups of 32 floats
                                                         uint32_t* __restrict__ out) {
  constexpr int PL = SIGN_ONLY ? 1 : BITS;
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  const int64_t total = n_groups32 * 32;
  const int64_t n_chunks = (n_groups32 + 1) / 2;  // 64 floats each, the last may be half
  const int64_t n_super = (n_chunks + CHUNKS - 1) / CHUNKS;
  for (int64_t sc = wave; sc < n_super; sc += n_waves) {
    const int64_t c0 = sc * CHUNKS;
    float v[CHUNKS];
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      const int64_t ch = c0 + c;
      v[c] = (ch * 64 + lane < total) ? y[ch * 64 + lane] : 0.f;
    }
    // lane L of the wave ends up holding output word L (and L+64, ... if any)
    // of this super-chunk: word index = (chunk*2 + half)*PL + plane
    constexpr int WORDS = CHUNKS * 2 * PL;
    constexpr int PER_LANE = (WORDS + 63) / 64;
    uint32_t mine[PER_LANE > 0 ? PER_LANE : 1];
#pragma unroll
    for (int q = 0; q < (PER_LANE > 0 ? PER_LANE : 1); ++q) mine[q] = 0u;
#pragma unroll
    for (int c = 0; c < CHUNKS; ++c) {
      uint64_t plane[PL > 0 ? PL : 1];
      if (SIGN_ONLY) {
        plane[0] = __ballot(v[c] >= 0.f);
      } else {
#pragma unroll
        for (int pl = 0; pl < PL; ++pl) plane[pl] = 0ull;
#pragma unroll
        for (int k = 0; k < (1 << BITS) - 1; ++k) {
          const uint64_t m = __ballot(v[c] >= cb.t[k]);
#pragma unroll
          for (int pl = 0; pl < PL; ++pl)
            if ((k & ((1 << pl) - 1)) == (1 << pl) - 1) plane[pl] ^= m;
        }
      }
#pragma unroll
      for (int pl = 0; pl < PL; ++pl) {
        const int w_lo = (c * 2 + 0) * PL + pl;
        const int w_hi = (c * 2 + 1) * PL + pl;
        if (lane == (w_lo & 63)) mine[w_lo >> 6] = (uint32_t)plane[pl];
        if (lane == (w_hi & 63)) mine[w_hi >> 6] = (uint32_t)(plane[pl] >> 32);
      }
    }
    const int64_t word0 = c0 * 2 * PL;
    const int64_t word_end = n_groups32 * PL;
#pragma unroll
    for (int q = 0; q < PER_LANE; ++q) {
      const int w = q * 64 + lane;
      if (w < WORDS && word0 + w < word_end) out[word0 + w] = mine[q];
    }
  }
}

template <int BITS>
__global__ __launch_bounds__(256) void stage_unpack_kernel(const Codebook cb, const uint32_t* __restrict__ idx,
                                                           const int64_t n_groups32,  // groups of 32 coords
                                                           float* __restrict__ out) {
  __shared__ float cent_s[16];
  if (threadIdx.x < 16) cent_s[threadIdx.x] = cb.c[threadIdx.x];
  __syncthreads();
  const int64_t total = n_groups32 * 32;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride) {
    const int64_t g = e >> 5;
    const int l = (int)(e & 31);
    uint32_t code = 0;
#pragma unroll
    for (int pl = 0; pl < BITS; ++pl) code |= ((idx[g * BITS + pl] >> l) & 1u) << pl;
    out[e] = cent_s[code];
  }
}

__global__ __launch_bounds__(256) void transpose_kernel(const int d, const float* __restrict__ in,
                                                        float* __restrict__ out) {
  __shared__ float tile[32][33];
  const int bx = blockIdx.x * 32, by = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  for (int r = ty; r < 32; r += 8)
    if (by + r < d && bx + tx < d) tile[r][tx] = in[(int64_t)(by + r) * d + bx + tx];
  __syncthreads();
  for (int r = ty; r < 32; r += 8)
    if (bx + r < d && by + tx < d) out[(int64_t)(bx + r) * d + by + tx] = tile[tx][r];
}

static int grid_for(int64_t work_items_per_wave_iter, int64_t n_items) {
  // enough workgroups to fill 256 CUs several times over, capped by the work
  int64_t waves = (n_items + work_items_per_wave_iter - 1) / work_items_per_wave_iter;
  int64_t blocks = (waves + 3) / 4;
  if (blocks > 256 * 16) blocks = 256 * 16;
  if (blocks < 1) blocks = 1;
  return (int)blocks;
}

template <int BITS>
static hipError_t pack_bits(const Codebook& cb, const float* y, int64_t groups, uint32_t* idx,
                            hipStream_t s) {
  hipLaunchKernelGGL((stage_pack_kernel<BITS, false>), dim3(grid_for(CHUNKS * 2, groups)), dim3(256), 0, s,
                     cb, y, groups, idx);
  return hipGetLastError();
}

hipError_t launch_stage_pack(const Codebook& cb, int d, const float* y, int64_t n, uint32_t* idx,
                             hipStream_t s) {
  const int64_t groups = n * (int64_t)(d / 32);
  if (groups == 0 || cb.bits == 0) return hipSuccess;
  switch (cb.bits) {
    case 1: return pack_bits<1>(cb, y, groups, idx, s);
    case 2: return pack_bits<2>(cb, y, groups, idx, s);
    case 3: return pack_bits<3>(cb, y, groups, idx, s);
    case 4: return pack_bits<4>(cb, y, groups, idx, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_stage_sign_pack(int d, const float* u, int64_t n, uint32_t* qjl, hipStream_t s) {
  const int64_t groups = n * (int64_t)(d / 32);
  if (groups == 0) return hipSuccess;
  Codebook cb = {};
  hipLaunchKernelGGL((stage_pack_kernel<1, true>), dim3(grid_for(CHUNKS * 2, groups)), dim3(256), 0, s, cb,
                     u, groups, qjl);
  return hipGetLastError();
}

template <int BITS>
static hipError_t unpack_bits(const Codebook& cb, const uint32_t* idx, int64_t groups, float* out,
                              hipStream_t s) {
  hipLaunchKernelGGL((stage_unpack_kernel<BITS>), dim3(grid_for(64 * 4, groups * 32)), dim3(256), 0, s, cb,
                     idx, groups, out);
  return hipGetLastError();
}

hipError_t launch_stage_unpack(const Codebook& cb, int d, const uint32_t* idx, int64_t n, float* out,
                               hipStream_t s) {
  const int64_t groups = n * (int64_t)(d / 32);
  if (groups == 0) return hipSuccess;
  switch (cb.bits) {
    case 0: return unpack_bits<0>(cb, idx, groups, out, s);
    case 1: return unpack_bits<1>(cb, idx, groups, out, s);
    case 2: return unpack_bits<2>(cb, idx, groups, out, s);
    case 3: return unpack_bits<3>(cb, idx, groups, out, s);
    case 4: return unpack_bits<4>(cb, idx, groups, out, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_transpose(int d, const float* in, float* out, hipStream_t s) {
  const int t = (d + 31) / 32;
  hipLaunchKernelGGL(transpose_kernel, dim3(t, t), dim3(256), 0, s, d, in, out);
  return hipGetLastError();
}

}  // namespace tq
