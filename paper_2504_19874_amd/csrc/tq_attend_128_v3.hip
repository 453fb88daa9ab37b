// Attention read-out at d = 128, value codes of Alg. 1 with 3-bit indices: the kernel variants for every kind of
// key code.
#include "tq_attend_128_kernel.h"

namespace tq {

TQ_ATTEND128_DECL(launch_attend128_v3) { return launch_attend128_vb<3, 0>(kb, kprod, ka, a, cf, cfh, n_groups, s); }

}  // namespace tq
