// Kernel-gradient kernels with 4 waves that share all columns and one to four map tiles (direct_wgrad_impl.h).
#include "direct_wgrad_impl.h"

namespace znn {

wgrad::WgradFn wgrad_kernel_h1a(int nj, int nt) { return wgrad::pick_nj<1, 4, true>(nj, nt); }

}  // namespace znn
