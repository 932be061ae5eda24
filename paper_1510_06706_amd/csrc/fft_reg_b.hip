// Register-resident strided FFT passes, extents 50, 54, 60, 64, 72 (see fft_reg_impl.h).
#include "fft_reg_impl.h"

namespace znn {

int fft_axis_reg_b(const RegAxis& P, int dir, hipStream_t s)
{
    switch (P.N) {
        case 50: return launch_n<50>(P, dir, s);
        case 54: return launch_n<54>(P, dir, s);
        case 60: return launch_n<60>(P, dir, s);
        case 64: return launch_n<64>(P, dir, s);
        case 72: return launch_n<72>(P, dir, s);
    }
    return fail(ZNN_EUNSUPPORTED, "no register FFT for extent %d", P.N);
}

}  // namespace znn
