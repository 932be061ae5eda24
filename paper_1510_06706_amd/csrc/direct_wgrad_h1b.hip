// Kernel-gradient kernels with 4 waves that share all columns and five to eight map tiles (direct_wgrad_impl.h).
#include "direct_wgrad_impl.h"

namespace znn {

wgrad::WgradFn wgrad_kernel_h1b(int nj, int nt) { return wgrad::pick_nj<1, 4, false>(nj, nt); }

}  // namespace znn
