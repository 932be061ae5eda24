// x and y passes in one launch, transform lengths 48, 50, 54, 60, 64 (see fft_xy_reg_impl.h).
#include "fft_xy_reg_impl.h"

namespace znn {

int fft_xy_reg_b(const XYFwd* F, const XYInv* B, int N, hipStream_t s)
{
    switch (N) {
        case 48: return launch_xy<48>(F, B, s);
        case 50: return launch_xy<50>(F, B, s);
        case 54: return launch_xy<54>(F, B, s);
        case 60: return launch_xy<60>(F, B, s);
        case 64: return launch_xy<64>(F, B, s);
    }
    return fail(ZNN_EUNSUPPORTED, "no fused x/y pass for extent %d", N);
}

}  // namespace znn
