// Direct-method kernels that walk the taps along x in groups of 11 (direct_mfma_impl.h).
#include "direct_mfma_impl.h"

namespace znn {

conv::ConvFn conv_kernel_u11(int nj, int nv, bool wl) { return conv::pick_kernel<11>(nj, nv, wl); }

}  // namespace znn
