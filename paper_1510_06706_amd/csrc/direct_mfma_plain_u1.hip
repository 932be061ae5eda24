// Direct-method kernels of full 16-map tiles only that walk the taps along x in groups of 1
// (direct_mfma_tail_impl.h).
#include "direct_mfma_tail_impl.h"

namespace znn {

conv::ConvFn conv_plain_kernel_u1(int nj, int nv, bool wl) { return conv::pick_tail_kernel<1, false>(nj, nv, wl); }

}  // namespace znn
