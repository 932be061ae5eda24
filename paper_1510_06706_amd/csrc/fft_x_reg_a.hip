// x-axis passes with the row's transform in registers, half lengths 8, 9, 10, 12, 15, 16, 18, 20, 24, 25, 27, 30, 32, 36 (see fft_x_reg_impl.h).
#include "fft_x_reg_impl.h"

namespace znn {

int fft_x_reg_a(const XRegR2C* F, const XRegC2R* B, int H, hipStream_t s)
{
    switch (H) {
        case 8: return launch_x<8>(F, B, s);
        case 9: return launch_x<9>(F, B, s);
        case 10: return launch_x<10>(F, B, s);
        case 12: return launch_x<12>(F, B, s);
        case 15: return launch_x<15>(F, B, s);
        case 16: return launch_x<16>(F, B, s);
        case 18: return launch_x<18>(F, B, s);
        case 20: return launch_x<20>(F, B, s);
        case 24: return launch_x<24>(F, B, s);
        case 25: return launch_x<25>(F, B, s);
        case 27: return launch_x<27>(F, B, s);
        case 30: return launch_x<30>(F, B, s);
        case 32: return launch_x<32>(F, B, s);
        case 36: return launch_x<36>(F, B, s);
    }
    return fail(ZNN_EUNSUPPORTED, "no register x pass for extent %d", 2 * H);
}

}  // namespace znn
