// Dispatch of the register-resident strided FFT passes (fft_reg_impl.h) over the translation
// units that instantiate them: every 5-smooth extent from 8 to 96.  Larger pencils do not
// fit the register file and take the LDS passes.
#include "znn_internal.h"

namespace znn {

int fft_axis_reg_a(const RegAxis& P, int dir, hipStream_t s);
int fft_axis_reg_b(const RegAxis& P, int dir, hipStream_t s);
int fft_axis_reg_c(const RegAxis& P, int dir, hipStream_t s);
int fft_axis_reg_d(const RegAxis& P, int dir, hipStream_t s);

bool fft_axis_reg_supported(int N)
{
    switch (N) {
        case 8: case 9: case 10: case 12: case 15: case 16: case 18: case 20: case 24: case 25: case 27: case 30: case 32: case 36: case 40: case 45: case 48: case 50: case 54: case 60: case 64: case 72: case 75: case 80: case 81: case 90: case 96:
            return true;
    }
    return false;
}

int fft_axis_reg(RegAxis P, int dir, hipStream_t s)
{
    // pencil index * L must stay below 2^32 for the multiply-high division
    // (and twice the pencil count, the thread index of the launches with two lanes per pencil, as well)
    if ((long)P.Ob * P.L * P.L >= 4294967296L || 2L * P.Ob * P.L >= 4294967296L || P.Oa > 65535)
        return fail(ZNN_EUNSUPPORTED, "too many pencils for one launch");
    P.fL = make_fastdiv((unsigned)P.L);
    switch (P.N) {
        case 8: case 9: case 10: case 12: case 15: case 16: case 18: case 20: case 24: case 25: case 27: case 30: case 32: case 36: case 40: case 45: case 48: return fft_axis_reg_a(P, dir, s);
        case 50: case 54: case 60: case 64: case 72: return fft_axis_reg_b(P, dir, s);
        case 75: case 80: case 81: return fft_axis_reg_c(P, dir, s);
        case 90: case 96: return fft_axis_reg_d(P, dir, s);
    }
    return fail(ZNN_EUNSUPPORTED, "no register FFT for extent %d", P.N);
}

}  // namespace znn
