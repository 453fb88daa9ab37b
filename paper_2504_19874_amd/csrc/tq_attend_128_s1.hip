// Attention read-out at d = 128, value codes of two instances of Alg. 1 over a split of the coordinates (Sec. 4.3)
// with 1 and 2 index bits: the kernel variants for every kind of key code.
#include "tq_attend_128_kernel.h"

namespace tq {

TQ_ATTEND128_DECL(launch_attend128_s1) { return launch_attend128_vb<1, 2>(kb, kprod, ka, a, cf, cfh, n_groups, s); }

}  // namespace tq
