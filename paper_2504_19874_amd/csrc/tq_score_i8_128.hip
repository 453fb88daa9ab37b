// Few queries per code at d = 128: the scoring kernel of tq_score_i8_128_body.h with the scores
// stored to memory.
#include "tq_score_i8_128_body.h"

namespace tq {

template <int BITS, bool PROD>
__global__ __launch_bounds__(512) void score_i8_128_kernel(const ScoreI8Args a) {
  __shared__ __attribute__((aligned(16))) uint2 expand_s[256 * I8_COPIES];
  extern __shared__ __attribute__((aligned(16))) unsigned char dyn_s[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int q = blockIdx.z * 4 + (lane >> 4);
  const bool out_live = q < a.q_per_group;
  float* const out0 = a.scores + ((int64_t)blockIdx.y * a.q_per_group + (out_live ? q : 0)) * a.lds +
                      ((int64_t)blockIdx.x * 8 + wave) * (16 * TILES_128) + (lane & 15);
  auto sink = [&](int t, float score, bool key_live) {
    if (out_live && key_live) out0[t * 16] = score;
  };
  score128_body<BITS, PROD>(a, expand_s, dyn_s, sink);
}

template <int BITS, bool PROD>
static hipError_t launch_128(const ScoreI8Args& a, int n_groups, hipStream_t s) {
  constexpr int lds = score128_lds(BITS);  // on top of the 64 KB table
  static_assert(I8_TABLE_BYTES + lds <= 160 * 1024, "LDS budget");
  const int64_t per_wg = 8 * 16 * TILES_128;
  const dim3 grid((unsigned)((a.n + per_wg - 1) / per_wg), n_groups, (a.q_per_group + 3) / 4);
  static LdsLimit lds_limit;  // per instantiation: the limit is raised once per device
  if (const hipError_t e = raise_lds_limit(lds_limit, reinterpret_cast<const void*>(&score_i8_128_kernel<BITS, PROD>), lds); e != hipSuccess) return e;
  hipLaunchKernelGGL((score_i8_128_kernel<BITS, PROD>), grid, dim3(512), lds, s, a);
  return hipGetLastError();
}

hipError_t launch_score_i8_128(int bits, bool prod, const ScoreI8Args& a, int n_groups, hipStream_t stream) {
  switch (bits * 2 + (prod ? 1 : 0)) {
    case 1: return launch_128<0, true>(a, n_groups, stream);
    case 2: return launch_128<1, false>(a, n_groups, stream);
    case 3: return launch_128<1, true>(a, n_groups, stream);
    case 4: return launch_128<2, false>(a, n_groups, stream);
    case 5: return launch_128<2, true>(a, n_groups, stream);
    case 6: return launch_128<3, false>(a, n_groups, stream);
    case 7: return launch_128<3, true>(a, n_groups, stream);
    case 8: return launch_128<4, false>(a, n_groups, stream);
    case 9: return launch_128<4, true>(a, n_groups, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace tq
