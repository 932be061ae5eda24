// Register-resident strided FFT passes, extents 8, 9, 10, 12, 15, 16, 18, 20, 24, 25, 27, 30, 32, 36, 40, 45, 48 (see fft_reg_impl.h).
#include "fft_reg_impl.h"

namespace znn {

int fft_axis_reg_a(const RegAxis& P, int dir, hipStream_t s)
{
    switch (P.N) {
        case 8: return launch_n<8>(P, dir, s);
        case 9: return launch_n<9>(P, dir, s);
        case 10: return launch_n<10>(P, dir, s);
        case 12: return launch_n<12>(P, dir, s);
        case 15: return launch_n<15>(P, dir, s);
        case 16: return launch_n<16>(P, dir, s);
        case 18: return launch_n<18>(P, dir, s);
        case 20: return launch_n<20>(P, dir, s);
        case 24: return launch_n<24>(P, dir, s);
        case 25: return launch_n<25>(P, dir, s);
        case 27: return launch_n<27>(P, dir, s);
        case 30: return launch_n<30>(P, dir, s);
        case 32: return launch_n<32>(P, dir, s);
        case 36: return launch_n<36>(P, dir, s);
        case 40: return launch_n<40>(P, dir, s);
        case 45: return launch_n<45>(P, dir, s);
        case 48: return launch_n<48>(P, dir, s);
    }
    return fail(ZNN_EUNSUPPORTED, "no register FFT for extent %d", P.N);
}

}  // namespace znn
