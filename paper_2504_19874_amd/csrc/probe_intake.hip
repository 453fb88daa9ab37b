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
