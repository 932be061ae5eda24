// Dispatch of the fused x/y passes (fft_xy_reg_impl.h) over the translation units that instantiate
// them: every even N up to 96 for which both N and N / 2 have register transforms.
#include "znn_internal.h"

namespace znn {

int fft_xy_reg_a(const XYFwd* F, const XYInv* B, int N, hipStream_t s);
int fft_xy_reg_b(const XYFwd* F, const XYInv* B, int N, hipStream_t s);
int fft_xy_reg_c(const XYFwd* F, const XYInv* B, int N, hipStream_t s);
int fft_xy_reg_d(const XYFwd* F, const XYInv* B, int N, hipStream_t s);

bool fft_xy_reg_supported(int N)
{
    return N % 2 == 0 && N >= 16 && N <= 96 && fft_axis_reg_supported(N) && fft_axis_reg_supported(N / 2);
}

static int dispatch(const XYFwd* F, const XYInv* B, int N, hipStream_t s)
{
    if (!fft_xy_reg_supported(N)) return fail(ZNN_EUNSUPPORTED, "no fused x/y pass for extent %d", N);
    if (N <= 40) return fft_xy_reg_a(F, B, N, s);
    if (N <= 64) return fft_xy_reg_b(F, B, N, s);
    if (N <= 80) return fft_xy_reg_c(F, B, N, s);
    return fft_xy_reg_d(F, B, N, s);
}

int fft_xy_fwd_reg(const XYFwd& P, int N, hipStream_t s) { return dispatch(&P, nullptr, N, s); }
int fft_xy_inv_reg(const XYInv& P, int N, hipStream_t s) { return dispatch(nullptr, &P, N, s); }

}  // namespace znn
