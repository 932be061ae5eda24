// x-axis passes with the row's transform in registers, half lengths 40, 45, 48, 50, 54, 60 (see fft_x_reg_impl.h).
#include "fft_x_reg_impl.h"

namespace znn {

int fft_x_reg_b(const XRegR2C* F, const XRegC2R* B, int H, hipStream_t s)
{
    switch (H) {
        case 40: return launch_x<40>(F, B, s);
        case 45: return launch_x<45>(F, B, s);
        case 48: return launch_x<48>(F, B, s);
        case 50: return launch_x<50>(F, B, s);
        case 54: return launch_x<54>(F, B, s);
        case 60: return launch_x<60>(F, B, s);
    }
    return fail(ZNN_EUNSUPPORTED, "no register x pass for extent %d", 2 * H);
}

}  // namespace znn
