// Few queries per code at d = 128: the scoring kernel of tq_score_i8_128_body.h with the scores
// stored to memory.
#include "tq_score_i8_128_body.h"

namespace tq {

template <int BITS, bool PROD, int TILES, int RTP = SCORE128_ROUND_TILES, int INFLIGHT = SCORE128_ROUNDS_AHEAD>
__global__ __launch_bounds__(512) void score_i8_128_kernel(const ScoreI8Args a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char dyn_s[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int q = blockIdx.z * 4 + (lane >> 4);
  const bool out_live = q < a.q_per_group;
  float* const out0 = a.scores + ((int64_t)blockIdx.y * a.q_per_group + (out_live ? q : 0)) * a.lds +
                      ((int64_t)blockIdx.x * 8 + wave) * (16 * TILES) + (lane & 15);
  auto sink = [&](int t, float score, bool key_live) {
    if (out_live && key_live) out0[t * 16] = score;
  };
  score128_body<BITS, PROD, TILES, RTP, INFLIGHT>(a, dyn_s, sink);
}

template <int BITS, bool PROD, int TILES, int RTP = SCORE128_ROUND_TILES, int INFLIGHT = SCORE128_ROUNDS_AHEAD>
static hipError_t launch_tiles(const ScoreI8Args& a, int n_groups, hipStream_t s) {
  constexpr int lds = score128_lds(BITS);
  static_assert(lds <= 160 * 1024, "LDS budget");
  const int64_t per_wg = 8 * 16 * TILES;
  const dim3 grid((unsigned)((a.n + per_wg - 1) / per_wg), n_groups, (a.q_per_group + 3) / 4);
  static LdsLimit lds_limit;  // per instantiation: the limit is raised once per device
  if (const hipError_t e = raise_lds_limit(lds_limit, reinterpret_cast<const void*>(&score_i8_128_kernel<BITS, PROD, TILES, RTP, INFLIGHT>), lds); e != hipSuccess) return e;
  hipLaunchKernelGGL((score_i8_128_kernel<BITS, PROD, TILES, RTP, INFLIGHT>), grid, dim3(512), lds, s, a);
  return hipGetLastError();
}

// Keys per workgroup: 2048, or 1024 / 512 where that still leaves compute units without a workgroup (a workgroup's
// fixed part, parameters and query rotation, is then paid by more of them, its tile phase shrinks).  8 heads of
// 16384 keys, 4 queries each, in a loop with the quantiser: 10.2 us with 512 keys per workgroup (256 workgroups)
// against 13.4 us with 2048 (64 workgroups); with every compute unit already taken (8 x 65536 keys) the smaller
// ranges lose: 18.8 / 26.0 us against 16.9.
template <int BITS, bool PROD>
static hipError_t launch_128(const ScoreI8Args& a, int n_groups, hipStream_t s) {
  const int64_t others = (int64_t)n_groups * ((a.q_per_group + 3) / 4), cus = device_cu_count();
  if (((a.n + 1023) / 1024) * others <= cus / 2) return launch_tiles<BITS, PROD, 4>(a, n_groups, s);
  if (((a.n + 2047) / 2048) * others <= cus / 2) return launch_tiles<BITS, PROD, 8>(a, n_groups, s);
  return launch_tiles<BITS, PROD, 16>(a, n_groups, s);
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
