// Register-resident strided FFT passes, extents 75, 80, 81 (see fft_reg_impl.h).
#include "fft_reg_impl.h"

namespace znn {

int fft_axis_reg_c(const RegAxis& P, int dir, hipStream_t s)
{
    switch (P.N) {
        case 75: return launch_n<75>(P, dir, s);
        case 80: return launch_n<80>(P, dir, s);
        case 81: return launch_n<81>(P, dir, s);
    }
    return fail(ZNN_EUNSUPPORTED, "no register FFT for extent %d", P.N);
}

}  // namespace znn
