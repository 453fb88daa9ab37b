// Attention read-out at d = 128, value codes of Alg. 2 with 1-bit indices plus the sign sketch: the kernel
// variants for every kind of key code.
#include "tq_attend_128_kernel.h"

namespace tq {

TQ_ATTEND128_DECL(launch_attend128_p1) { return launch_attend128_vb<1, 1>(kb, kprod, ka, a, cf, cfh, n_groups, s); }

}  // namespace tq
