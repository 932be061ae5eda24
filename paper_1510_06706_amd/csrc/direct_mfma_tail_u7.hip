// Direct-method kernels with an 8-map block behind the full tiles that walk the taps along x in
// groups of 7 (direct_mfma_tail_impl.h).
#include "direct_mfma_tail_impl.h"

namespace znn {

conv::ConvFn conv_tail_kernel_u7(int nj, int nv, bool wl) { return conv::pick_tail_kernel<7, true>(nj, nv, wl); }

}  // namespace znn
