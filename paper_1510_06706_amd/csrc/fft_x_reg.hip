// Dispatch of the x-axis passes with register-resident rows (fft_x_reg_impl.h) over the translation
// units that instantiate them: N = 2 H for every 5-smooth H from 8 to 96.
#include "znn_internal.h"

namespace znn {

int fft_x_reg_a(const XRegR2C* F, const XRegC2R* B, int H, hipStream_t s);
int fft_x_reg_b(const XRegR2C* F, const XRegC2R* B, int H, hipStream_t s);
int fft_x_reg_c(const XRegR2C* F, const XRegC2R* B, int H, hipStream_t s);
int fft_x_reg_d(const XRegR2C* F, const XRegC2R* B, int H, hipStream_t s);

bool fft_x_reg_supported(int N) { return N % 2 == 0 && fft_axis_reg_supported(N / 2); }

static int dispatch(const XRegR2C* F, const XRegC2R* B, int N, hipStream_t s)
{
    if (!fft_x_reg_supported(N)) return fail(ZNN_EUNSUPPORTED, "no register x pass for extent %d", N);
    const int H = N / 2;
    if (H <= 36) return fft_x_reg_a(F, B, H, s);
    if (H <= 60) return fft_x_reg_b(F, B, H, s);
    if (H <= 80) return fft_x_reg_c(F, B, H, s);
    return fft_x_reg_d(F, B, H, s);
}

int fft_x_r2c_reg(const XRegR2C& P, int N, hipStream_t s) { return dispatch(&P, nullptr, N, s); }
int fft_x_c2r_reg(const XRegC2R& P, int N, hipStream_t s) { return dispatch(nullptr, &P, N, s); }

}  // namespace znn
