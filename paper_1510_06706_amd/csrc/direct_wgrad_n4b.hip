// Kernel-gradient kernels with 4 waves with their own columns each and five to eight map tiles (direct_wgrad_impl.h).
#include "direct_wgrad_impl.h"

namespace znn {

wgrad::WgradFn wgrad_kernel_n4b(int nj, int nt) { return wgrad::pick_nj<4, 1, false>(nj, nt); }

}  // namespace znn
