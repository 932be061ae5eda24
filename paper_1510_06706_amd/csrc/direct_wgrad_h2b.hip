// Kernel-gradient kernels with 8 waves in two column sets and five to eight map tiles (direct_wgrad_impl.h).
#include "direct_wgrad_impl.h"

namespace znn {

wgrad::WgradFn wgrad_kernel_h2b(int nj, int nt) { return wgrad::pick_nj<2, 4, false>(nj, nt); }

}  // namespace znn
