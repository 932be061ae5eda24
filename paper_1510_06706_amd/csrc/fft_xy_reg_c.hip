// x and y passes in one launch, transform lengths 72, 80 (see fft_xy_reg_impl.h).
#include "fft_xy_reg_impl.h"

namespace znn {

int fft_xy_reg_c(const XYFwd* F, const XYInv* B, int N, hipStream_t s)
{
    switch (N) {
        case 72: return launch_xy<72>(F, B, s);
        case 80: return launch_xy<80>(F, B, s);
    }
    return fail(ZNN_EUNSUPPORTED, "no fused x/y pass for extent %d", N);
}

}  // namespace znn
