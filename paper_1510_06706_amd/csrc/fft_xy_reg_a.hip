// x and y passes in one launch, transform lengths 16, 18, 20, 24, 30, 32, 36, 40 (see fft_xy_reg_impl.h).
#include "fft_xy_reg_impl.h"

namespace znn {

int fft_xy_reg_a(const XYFwd* F, const XYInv* B, int N, hipStream_t s)
{
    switch (N) {
        case 16: return launch_xy<16>(F, B, s);
        case 18: return launch_xy<18>(F, B, s);
        case 20: return launch_xy<20>(F, B, s);
        case 24: return launch_xy<24>(F, B, s);
        case 30: return launch_xy<30>(F, B, s);
        case 32: return launch_xy<32>(F, B, s);
        case 36: return launch_xy<36>(F, B, s);
        case 40: return launch_xy<40>(F, B, s);
    }
    return fail(ZNN_EUNSUPPORTED, "no fused x/y pass for extent %d", N);
}

}  // namespace znn
