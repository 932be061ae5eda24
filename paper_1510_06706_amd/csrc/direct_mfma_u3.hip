// Direct-method kernels that walk the taps along x in groups of 3 (direct_mfma_impl.h).
#include "direct_mfma_impl.h"

namespace znn {

conv::ConvFn conv_kernel_u3(int nj, int nv, bool wl) { return conv::pick_kernel<3>(nj, nv, wl); }

}  // namespace znn
