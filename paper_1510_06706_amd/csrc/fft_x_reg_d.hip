// x-axis passes with the row's transform in registers, half lengths 81, 90, 96 (see fft_x_reg_impl.h).
#include "fft_x_reg_impl.h"

namespace znn {

int fft_x_reg_d(const XRegR2C* F, const XRegC2R* B, int H, hipStream_t s)
{
    switch (H) {
        case 81: return launch_x<81>(F, B, s);
        case 90: return launch_x<90>(F, B, s);
        case 96: return launch_x<96>(F, B, s);
    }
    return fail(ZNN_EUNSUPPORTED, "no register x pass for extent %d", 2 * H);
}

}  // namespace znn
