// x-axis passes with the row's transform in registers, half lengths 64, 72, 75, 80 (see fft_x_reg_impl.h).
#include "fft_x_reg_impl.h"

namespace znn {

int fft_x_reg_c(const XRegR2C* F, const XRegC2R* B, int H, hipStream_t s)
{
    switch (H) {
        case 64: return launch_x<64>(F, B, s);
        case 72: return launch_x<72>(F, B, s);
        case 75: return launch_x<75>(F, B, s);
        case 80: return launch_x<80>(F, B, s);
    }
    return fail(ZNN_EUNSUPPORTED, "no register x pass for extent %d", 2 * H);
}

}  // namespace znn
