// Kernel-gradient kernels with 4 waves with their own columns each and one to four map tiles (direct_wgrad_impl.h).
#include "direct_wgrad_impl.h"

namespace znn {

wgrad::WgradFn wgrad_kernel_n4a(int nj, int nt) { return wgrad::pick_nj<4, 1, true>(nj, nt); }

}  // namespace znn
