// Kernel-gradient kernels with 8 waves in two column sets and one to four map tiles (direct_wgrad_impl.h).
#include "direct_wgrad_impl.h"

namespace znn {

wgrad::WgradFn wgrad_kernel_h2a(int nj, int nt) { return wgrad::pick_nj<2, 4, true>(nj, nt); }

}  // namespace znn
