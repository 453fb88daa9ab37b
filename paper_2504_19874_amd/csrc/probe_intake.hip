// Measurement aid, not part of the quantiser: how fast one workgroup per compute unit can take in a
// given number of bytes, which is what bounds the few-query scoring kernel (every workgroup there
// needs the codes of its own keys plus the two 64 KB parameter matrices that all workgroups read).
// A workgroup of 512 threads issues NS 16-byte loads per thread from a region every workgroup
// shares and NP from a region of its own, all before the first use, folds them into one word and
// stores it.  Built into its own small library; only the kernel benchmark loads it.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int NS, int NP>
__global__ __launch_bounds__(512) void intake_kernel(const u32x4* shared, const u32x4* own, uint32_t* out) {
  const int tid = threadIdx.x;
  u32x4 s[NS > 0 ? NS : 1], p[NP > 0 ? NP : 1];
  const u32x4* const mine = own + (size_t)blockIdx.x * NP * 512;
#pragma unroll
  for (int i = 0; i < NS; ++i) s[i] = shared[i * 512 + tid];
#pragma unroll
  for (int i = 0; i < NP; ++i) p[i] = mine[i * 512 + tid];
  uint32_t acc = 0;
#pragma unroll
  for (int i = 0; i < NS; ++i) acc ^= s[i][0] ^ s[i][1] ^ s[i][2] ^ s[i][3];
#pragma unroll
  for (int i = 0; i < NP; ++i) acc ^= p[i][0] ^ p[i][1] ^ p[i][2] ^ p[i][3];
  out[(size_t)blockIdx.x * 512 + tid] = acc;
}


// When the loads of a wavefront come back: the same intake (NP 16-byte loads per thread of the workgroup's own
// region, all issued before the first wait), with the constant-rate clock read at the start and after each
// "at most NP - k loads outstanding" wait, k = 1 .. NP.  Lane 0 of every wavefront writes its NP + 1 readings to
// stamps[(workgroup * 8 + wavefront) * 16 + k].
template <int N>
__device__ __forceinline__ void wait_outstanding() {  // s_waitcnt vmcnt(N), other counters left alone
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}
template <int NP, int K>
struct ArrivalSteps {
  static __device__ __forceinline__ void run(uint64_t* t) {
    if constexpr (K <= NP) {
      wait_outstanding<NP - K>();
      t[K] = wall_clock64();
      ArrivalSteps<NP, K + 1>::run(t);
    }
  }
};

template <int NP>
__global__ __launch_bounds__(512) void arrival_kernel(const u32x4* own, uint32_t* out, uint64_t* stamps) {
  const int tid = threadIdx.x;
  uint64_t t[NP + 1];
  t[0] = wall_clock64();
  u32x4 p[NP];
  const u32x4* const mine = own + (size_t)blockIdx.x * NP * 512;
#pragma unroll
  for (int i = 0; i < NP; ++i) p[i] = mine[i * 512 + tid];
  ArrivalSteps<NP, 1>::run(t);
  uint32_t acc = 0;
#pragma unroll
  for (int i = 0; i < NP; ++i) acc ^= p[i][0] ^ p[i][1] ^ p[i][2] ^ p[i][3];
  out[(size_t)blockIdx.x * 512 + tid] = acc;
  if ((tid & 63) == 0) {
#pragma unroll
    for (int k = 0; k <= NP; ++k) stamps[((size_t)blockIdx.x * 8 + (tid >> 6)) * 16 + k] = t[k];
  }
}

template <int NS, int NP>
int launch(const void* shared, const void* own, void* out, int workgroups, hipStream_t st) {
  intake_kernel<NS, NP><<<workgroups, 512, 0, st>>>(static_cast<const u32x4*>(shared), static_cast<const u32x4*>(own),
                                                   static_cast<uint32_t*>(out));
  return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace

// shared: shared_kb KB read by every workgroup; own: workgroups * own_kb KB, own_kb KB per workgroup;
// out: workgroups * 512 words.  All device pointers.  (shared_kb, own_kb) must be one of the
// combinations below (8 KB = one 16-byte load per thread); returns 0 on success, 2 for any other.
extern "C" int tq_probe_intake(const void* shared, int shared_kb, const void* own, int own_kb, void* out,
                               int workgroups, void* stream) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (shared == nullptr || own == nullptr || out == nullptr || workgroups <= 0) return 2;
#define CASE(S, P) \
  if (shared_kb == 8 * S && own_kb == 8 * P) return launch<S, P>(shared, own, out, workgroups, st);
  CASE(0, 1) CASE(0, 7) CASE(0, 14) CASE(0, 22) CASE(0, 30)
  CASE(8, 0) CASE(16, 0) CASE(8, 14) CASE(16, 14) CASE(4, 14) CASE(16, 7) CASE(8, 7)
#undef CASE
  return 2;
}

// own: workgroups * 112 KB; out: workgroups * 512 words; stamps: workgroups * 8 * 16 64-bit words (14 loads per
// thread: readings 0 .. 14 of each wavefront, 100 MHz clock).  All device pointers.  Returns 0 on success.
extern "C" int tq_probe_arrival(const void* own, void* out, void* stamps, int workgroups, void* stream) {
  if (own == nullptr || out == nullptr || stamps == nullptr || workgroups <= 0) return 2;
  arrival_kernel<14><<<workgroups, 512, 0, static_cast<hipStream_t>(stream)>>>(
      static_cast<const u32x4*>(own), static_cast<uint32_t*>(out), static_cast<uint64_t*>(stamps));
  return hipGetLastError() == hipSuccess ? 0 : 1;
}
