// x and y passes in one launch, transform lengths 90, 96 (see fft_xy_reg_impl.h).
#include "fft_xy_reg_impl.h"

namespace znn {

int fft_xy_reg_d(const XYFwd* F, const XYInv* B, int N, hipStream_t s)
{
    switch (N) {
        case 90: return launch_xy<90>(F, B, s);
        case 96: return launch_xy<96>(F, B, s);
    }
    return fail(ZNN_EUNSUPPORTED, "no fused x/y pass for extent %d", N);
}

}  // namespace znn
