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
#include <utility>

#include "tq_internal.h"

namespace tq {

constexpr int CHUNKS = 8;  // 64-coordinate chunks per wavefront iteration

typedef float f32x4 __attribute__((ext_vector_type(4)));

// put a wave-uniform 32-bit value into one lane of a vector register.  The value
// usually comes straight from a vector compare (VALU-written scalar register);
// v_writelane_b32 must not read such a register in the very next cycles, and the
// compiler does not track hazards inside inline asm, so the value is first
// copied by a scalar move (scalar reads of VALU-written registers are
// interlocked by hardware, and scalar-written registers are safe to read).
template <int LANE>
__device__ __forceinline__ int write_lane(int old, uint32_t uniform_value) {
  uint32_t tmp;
  asm volatile("s_mov_b32 %1, %2\n\tv_writelane_b32 %0, %1, %3"
               : "+v"(old), "=&s"(tmp)
               : "s"(uniform_value), "n"(LANE));
  return old;
}

// output word W of a super-chunk lives in lane W%64 of register W/64
template <int W, int N>
__device__ __forceinline__ void put_word(int (&mine)[N], uint32_t uniform_value) {
  mine[W >> 6] = write_lane<(W & 63)>(mine[W >> 6], uniform_value);
}

template <int C, int PL, int N, int... P>
__device__ __forceinline__ void route_planes(std::integer_sequence<int, P...>, const uint64_t (&plane)[PL],
                                             int (&mine)[N]) {
  ((put_word<(C * 2 + 0) * PL + P>(mine, (uint32_t)plane[P]),
    put_word<(C * 2 + 1) * PL + P>(mine, (uint32_t)(plane[P] >> 32))),
   ...);
}

// SYM: the table is symmetric about zero (c[i] = -c[K-1-i], middle boundary 0; checked by the launcher), so the
// bucket is found on |v| with half the compares.  With H = K / 2 magnitude buckets a coordinate v >= 0 in magnitude
// bucket m has index H + m and a negative one H - 1 - m: the low planes are m or its complement, the top plane is
// the sign compare.  "On a boundary, the upper cell" is |v| >= T for v >= 0 but |v| > T for v < 0, so negative
// values are compared one ulp smaller (a subtract-with-borrow whose borrow is the sign mask; -0 counts as >= 0).
template <int BITS, bool SIGN_ONLY, bool SYM, int C, int N>
__device__ __forceinline__ void pack_chunk(const Codebook& cb, const float v, int (&mine)[N]) {
  constexpr int PL = SIGN_ONLY ? 1 : BITS;
  uint64_t plane[PL];
  if (SIGN_ONLY) {
    plane[0] = __ballot(v >= 0.f);
  } else if (SYM) {
    constexpr int H = 1 << (BITS - 1);
    const uint64_t pos = __ballot(v >= 0.f);
    uint32_t av = __float_as_uint(v) & 0x7fffffffu;
    {
      uint64_t borrow_out;
      const uint64_t neg = ~pos;
      asm("v_subb_co_u32 %0, %1, %2, 0, %3" : "=v"(av), "=s"(borrow_out) : "v"(av), "s"(neg));
    }
    const float avf = __uint_as_float(av);
#pragma unroll
    for (int pl = 0; pl < PL; ++pl) plane[pl] = 0ull;
#pragma unroll
    for (int j = 0; j < H - 1; ++j) {
      const uint64_t m = __ballot(avf >= cb.t[H + j]);
#pragma unroll
      for (int pl = 0; pl < PL - 1; ++pl)
        if ((j & ((1 << pl) - 1)) == (1 << pl) - 1) plane[pl] ^= m;
    }
#pragma unroll
    for (int pl = 0; pl < PL - 1; ++pl) plane[pl] ^= ~pos;
    plane[PL - 1] = pos;
  } else {
#pragma unroll
    for (int pl = 0; pl < PL; ++pl) plane[pl] = 0ull;
#pragma unroll
    for (int k = 0; k < (1 << BITS) - 1; ++k) {
      const uint64_t m = __ballot(v >= cb.t[k]);
#pragma unroll
      for (int pl = 0; pl < PL; ++pl)
        if ((k & ((1 << pl) - 1)) == (1 << pl) - 1) plane[pl] ^= m;
    }
  }
  // the masks are wave-uniform scalars: drop each 32-bit half into the lane that stores it
  route_planes<C, PL>(std::make_integer_sequence<int, PL>{}, plane, mine);
  __builtin_amdgcn_sched_barrier(0);  // one chunk's masks at a time (scalar register pressure)
}

template <int BITS, bool SIGN_ONLY, bool SYM, int N, int... C>
__device__ __forceinline__ void pack_chunks(std::integer_sequence<int, C...>, const Codebook& cb,
                                            const float (&v)[CHUNKS], int (&mine)[N]) {
  (pack_chunk<BITS, SIGN_ONLY, SYM, C>(cb, v[C], mine), ...);
}

template <int BITS, bool SIGN_ONLY, bool SYM = false>
__global__ __launch_bounds__(256) void stage_pack_kernel(const Codebook cb, const float* __restrict__ y,
                                                         const int64_t n_groups32,  // groups of 32 floats
                                                         uint32_t* __restrict__ out) {
  constexpr int PL = SIGN_ONLY ? 1 : BITS;
  constexpr int WORDS = CHUNKS * 2 * PL;       // output words per super-chunk
  constexpr int PER_LANE = (WORDS + 63) / 64;  // lane L holds word L (and L+64 ...)
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
  const int64_t total = n_groups32 * 32;
  const int64_t n_chunks = (n_groups32 + 1) / 2;  // 64 floats each, the last may be half
  const int64_t n_super = (n_chunks + CHUNKS - 1) / CHUNKS;
  for (int64_t sc = wave; sc < n_super; sc += n_waves) {
    const int64_t c0 = sc * CHUNKS;
    const float* src = y + c0 * 64 + lane;
    float v[CHUNKS];
    if ((c0 + CHUNKS) * 64 <= total) {  // whole super-chunk in range: no per-load guards
#pragma unroll
      for (int c = 0; c < CHUNKS; ++c) v[c] = __builtin_nontemporal_load(src + c * 64);
    } else {
#pragma unroll
      for (int c = 0; c < CHUNKS; ++c) v[c] = ((c0 + c) * 64 + lane < total) ? src[c * 64] : 0.f;
    }
    int mine[PER_LANE];
#pragma unroll
    for (int q = 0; q < PER_LANE; ++q) mine[q] = 0;
    pack_chunks<BITS, SIGN_ONLY, SYM>(std::make_integer_sequence<int, CHUNKS>{}, cb, v, mine);
    const int64_t word0 = c0 * 2 * PL;
    const int64_t word_end = n_groups32 * PL;
#pragma unroll
    for (int q = 0; q < PER_LANE; ++q) {
      const int w = q * 64 + lane;
      if (w < WORDS && word0 + w < word_end) out[word0 + w] = (uint32_t)mine[q];
    }
  }
}

// Each lane produces 4 consecutive coordinates (one 16-byte store); the 8 lanes
// that share a 32-coordinate group read the same plane words.
template <int BITS>
__global__ __launch_bounds__(256) void stage_unpack_kernel(const Codebook cb, const uint32_t* __restrict__ idx,
                                                           const int64_t n_groups32,  // groups of 32 coords
                                                           float* __restrict__ out) {
  __shared__ float cent_s[16];
  if (threadIdx.x < 16) cent_s[threadIdx.x] = cb.c[threadIdx.x];
  __syncthreads();
  const int64_t n_quads = n_groups32 * 8;
  constexpr int U = 4;
  const int64_t stride = 256;  // a workgroup's U stores per thread cover one contiguous 16 KB (8 or 32 KB: slower)
  for (int64_t q0 = (int64_t)blockIdx.x * (256 * U) + threadIdx.x; q0 < n_quads; q0 += (int64_t)gridDim.x * (256 * U)) {
    uint32_t w[U][BITS > 0 ? BITS : 1];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t qd = q0 + u * stride;
      if (qd < n_quads) {
#pragma unroll
        for (int pl = 0; pl < BITS; ++pl) w[u][pl] = idx[(qd >> 3) * BITS + pl] >> (4 * (int)(qd & 7));
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t qd = q0 + u * stride;
      if (qd < n_quads) {
        // four bucket numbers at once: a plane's 4 bits are spread to one bit per byte by a multiply (bit i
        // lands at 8 i), the planes are merged so that byte k holds 4 * code_k, the byte offset into the table
        uint32_t x = 0u;
#pragma unroll
        for (int pl = 0; pl < BITS; ++pl) x |= (((w[u][pl] & 0xFu) * 0x00204081u) & 0x01010101u) << (pl + 2);
        float e[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
          e[k] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(cent_s) + ((x >> (8 * k)) & 0xFFu));
        f32x4 o4 = {e[0], e[1], e[2], e[3]};
        __builtin_nontemporal_store(o4, reinterpret_cast<f32x4*>(out) + qd);
      }
    }
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
  // One pass of the kernel's loop per wavefront (the loop only serves inputs beyond 2^30 workgroups): workgroups
  // that the hardware hands out in order, each on its own contiguous 16 KB, stream faster than 4096 persistent
  // ones striding over the array (C4-shaped sign packing 6.5 against 5.4 TB/s, unpacking 5.2 against 4.2).
  int64_t waves = (n_items + work_items_per_wave_iter - 1) / work_items_per_wave_iter;
  int64_t blocks = (waves + 3) / 4;
  if (blocks > (1 << 30)) blocks = 1 << 30;
  if (blocks < 1) blocks = 1;
  return (int)blocks;
}

template <int BITS>
static hipError_t pack_bits(const Codebook& cb, const float* y, int64_t groups, uint32_t* idx,
                            hipStream_t s) {
  // from 3 bits on, a table that is symmetric about zero (what the Lloyd-Max solution is) is decided on |y|
  bool sym = BITS >= 3;
  for (int i = 0; sym && i < (1 << BITS); ++i) sym = cb.c[i] == -cb.c[(1 << BITS) - 1 - i];
  for (int j = 0; sym && j + 1 < (1 << BITS); ++j) sym = cb.t[j] == -cb.t[(1 << BITS) - 2 - j];
  if (sym)
    hipLaunchKernelGGL((stage_pack_kernel<BITS, false, (BITS >= 3)>), dim3(grid_for(CHUNKS * 2, groups)), dim3(256), 0, s,
                       cb, y, groups, idx);
  else
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
  const int64_t wgs = (groups * 8 + 1023) / 1024;
  hipLaunchKernelGGL((stage_unpack_kernel<BITS>), dim3((unsigned)(wgs < (1 << 30) ? wgs : (1 << 30))), dim3(256), 0, s, cb,
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
