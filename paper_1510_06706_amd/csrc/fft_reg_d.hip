// Register-resident strided FFT passes, extents 90, 96 (see fft_reg_impl.h).
#include "fft_reg_impl.h"

namespace znn {

int fft_axis_reg_d(const RegAxis& P, int dir, hipStream_t s)
{
    switch (P.N) {
        case 90: return launch_n<90>(P, dir, s);
        case 96: return launch_n<96>(P, dir, s);
    }
    return fail(ZNN_EUNSUPPORTED, "no register FFT for extent %d", P.N);
}

}  // namespace znn
