// Attention read-out at d = 128 on the integer matrix cores: which kernel variant a call takes
// (the kernel itself is in tq_attend_128_kernel.h).
#include <cstring>

#include "tq_attend_128_kernel.h"

namespace tq {

int attend128_chunks(int64_t n) { return (int)((n + AT_CHUNK - 1) / AT_CHUNK); }

// value codes the kernel covers: d = 128, tables symmetric about zero; codes of Alg. 1 with 1..4 index bits,
// codes of Alg. 2 with 0..2, or two instances of Alg. 1 (cb_hi != NULL) with 1 + 2 or 2 + 3
bool attend128_applicable(int d, bool prod, const Codebook& cb, const Codebook* cb_hi) {
  float coef[16];
  if (d != 128 || !i8_coefficients(cb.bits, cb, coef)) return false;
  if (cb_hi != nullptr)
    return !prod && cb.bits >= 1 && cb.bits <= 2 && cb_hi->bits == cb.bits + 1 && i8_coefficients(cb_hi->bits, *cb_hi, coef);
  return cb.bits >= (prod ? 0 : 1) && cb.bits <= (prod ? 2 : 4);
}

// ka == nullptr: logits from a.scores; otherwise the scoring body runs in the same kernel on key codes of
// kb index bits (kprod: with the sign sketch)
hipError_t launch_attend128(int kb, bool kprod, const ScoreI8Args* ka, bool vprod, const AttendArgs& a, int n_groups,
                            hipStream_t s) {
  if (a.nchunks == 0 || n_groups == 0 || a.q_per_group == 0) return hipSuccess;
  ScoreI8Args none;
  std::memset(&none, 0, sizeof(none));
  const ScoreI8Args& k = ka != nullptr ? *ka : none;
  if (ka == nullptr) kb = -1;
  AttendCoefs cf, cfh;
  std::memset(&cfh, 0, sizeof(cfh));
  if (a.d != 128 || !i8_coefficients(a.cb.bits, a.cb, cf.c)) return hipErrorInvalidValue;
  if (a.gs_hi > 0) {
    if (vprod || !i8_coefficients(a.cb_hi.bits, a.cb_hi, cfh.c)) return hipErrorInvalidValue;
    switch (a.cb.bits) {
      case 1: return launch_attend128_s1(kb, kprod, k, a, cf, cfh, n_groups, s);
      case 2: return launch_attend128_s2(kb, kprod, k, a, cf, cfh, n_groups, s);
      default: return hipErrorInvalidValue;
    }
  }
  if (vprod) {
    switch (a.cb.bits) {
      case 0: return launch_attend128_p0(kb, kprod, k, a, cf, cfh, n_groups, s);
      case 1: return launch_attend128_p1(kb, kprod, k, a, cf, cfh, n_groups, s);
      case 2: return launch_attend128_p2(kb, kprod, k, a, cf, cfh, n_groups, s);
      default: return hipErrorInvalidValue;
    }
  }
  switch (a.cb.bits) {
    case 1: return launch_attend128_v1(kb, kprod, k, a, cf, cfh, n_groups, s);
    case 2: return launch_attend128_v2(kb, kprod, k, a, cf, cfh, n_groups, s);
    case 3: return launch_attend128_v3(kb, kprod, k, a, cf, cfh, n_groups, s);
    case 4: return launch_attend128_v4(kb, kprod, k, a, cf, cfh, n_groups, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace tq
