// Kernel-gradient kernels with 8 waves with their own columns each and one to four map tiles (direct_wgrad_impl.h).
#include "direct_wgrad_impl.h"

namespace znn {

wgrad::WgradFn wgrad_kernel_n8a(int nj, int nt) { return wgrad::pick_nj<8, 1, true>(nj, nt); }

}  // namespace znn
