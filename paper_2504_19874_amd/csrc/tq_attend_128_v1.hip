// Attention read-out at d = 128, value codes with 1-bit indices: the kernel variants for every kind of key code.
#include "tq_attend_128_kernel.h"

namespace tq {

hipError_t launch_attend128_v1(int kb, bool kprod, const ScoreI8Args& ka, const AttendArgs& a, const AttendCoefs& cf,
                               int n_groups, hipStream_t s) {
  return launch_attend128_vb<1>(kb, kprod, ka, a, cf, n_groups, s);
}

}  // namespace tq
