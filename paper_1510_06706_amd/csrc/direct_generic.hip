// Direct method, shape-agnostic kernels: one thread per result element, plain
// fp32 FMAs.  They cover every legal descriptor and serve the shapes the tiled
// MFMA kernels do not take (tiny fan widths, very large kernels).
#include "znn_internal.h"

namespace znn {

// Forward pass (Section 2): out[j][p] = sum_i sum_a w[j][i][a] * in[i][p + s(k-1-a)].
__global__ void __launch_bounds__(256)
k_direct_fwd_generic(Geom g, const float* __restrict__ in, const float* __restrict__ w,
                     float* __restrict__ out)
{
    const long ovol = g.ovol();
    const long p = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const int j = blockIdx.y;
    if (p >= ovol) return;
    const int x = (int)(p % g.ox);
    const int y = (int)((p / g.ox) % g.oy);
    const int z = (int)(p / ((long)g.ox * g.oy));
    const long nvol = g.nvol(), kvol = g.kvol();
    float acc = 0.f;
    for (int i = 0; i < g.f; ++i) {
        const float* img = in + i * nvol;
        const float* ker = w + ((long)j * g.f + i) * kvol;
        for (int a = 0; a < g.kz; ++a)
            for (int b = 0; b < g.ky; ++b) {
                const float* row = img + ((long)(z + g.spz * (g.kz - 1 - a)) * g.ny + (y + g.spy * (g.ky - 1 - b))) * g.nx +
                                   x + g.spx * (g.kx - 1);
                const float* kr = ker + ((long)a * g.ky + b) * g.kx;
                for (int c = 0; c < g.kx; ++c) acc = fmaf(kr[c], row[-c * g.spx], acc);
            }
    }
    out[(long)j * ovol + p] = acc;
}

// Backward pass (Section 3.1): gin[i][q] = sum_j sum_a w[j][i][a] * gout[j][q - s(k-1-a)].
__global__ void __launch_bounds__(256)
k_direct_bwd_generic(Geom g, const float* __restrict__ gout, const float* __restrict__ w,
                     float* __restrict__ gin)
{
    const long nvol = g.nvol();
    const long q = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const int i = blockIdx.y;
    if (q >= nvol) return;
    const int x = (int)(q % g.nx);
    const int y = (int)((q / g.nx) % g.ny);
    const int z = (int)(q / ((long)g.nx * g.ny));
    const long ovol = g.ovol(), kvol = g.kvol();
    float acc = 0.f;
    for (int j = 0; j < g.fo; ++j) {
        const float* gimg = gout + j * ovol;
        const float* ker = w + ((long)j * g.f + i) * kvol;
        for (int a = 0; a < g.kz; ++a) {
            const int gz = z - g.spz * (g.kz - 1 - a);
            if (gz < 0 || gz >= g.oz) continue;
            for (int b = 0; b < g.ky; ++b) {
                const int gy = y - g.spy * (g.ky - 1 - b);
                if (gy < 0 || gy >= g.oy) continue;
                const float* kr = ker + ((long)a * g.ky + b) * g.kx;
                const float* row = gimg + ((long)gz * g.oy + gy) * g.ox;
                for (int c = 0; c < g.kx; ++c) {
                    const int gx = x - g.spx * (g.kx - 1 - c);
                    if (gx >= 0 && gx < g.ox) acc = fmaf(kr[c], row[gx], acc);
                }
            }
        }
    }
    gin[(long)i * nvol + q] = acc;
}

// Kernel gradient (Section 3.2): gw[j][i][a] = sum_p gout[j][p] * in[i][p + s(k-1-a)].
// One block per (edge, tap); fixed-shape tree reduction, so the result does not
// depend on timing.
__global__ void __launch_bounds__(256)
k_direct_wgrad_generic(Geom g, const float* __restrict__ in, const float* __restrict__ gout,
                       float* __restrict__ gw)
{
    __shared__ float red[256];
    const long kvol = g.kvol(), ovol = g.ovol(), nvol = g.nvol();
    const long e = blockIdx.x / kvol;
    const int tap = (int)(blockIdx.x % kvol);
    const int j = (int)(e / g.f), i = (int)(e % g.f);
    const int c = tap % g.kx, b = (tap / g.kx) % g.ky, a = tap / (g.kx * g.ky);
    const float* img = in + i * nvol;
    const float* gimg = gout + j * ovol;
    const long shift = ((long)g.spz * (g.kz - 1 - a) * g.ny + g.spy * (g.ky - 1 - b)) * g.nx + g.spx * (g.kx - 1 - c);
    float acc = 0.f;
    for (long p = threadIdx.x; p < ovol; p += 256) {
        const int x = (int)(p % g.ox);
        const int y = (int)((p / g.ox) % g.oy);
        const int z = (int)(p / ((long)g.ox * g.oy));
        acc = fmaf(gimg[p], img[((long)z * g.ny + y) * g.nx + x + shift], acc);
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) gw[blockIdx.x] = red[0];
}

int direct_fwd_generic(const Geom& g, const float* in, const float* w, float* out, hipStream_t s)
{
    dim3 grid((unsigned)((g.ovol() + 255) / 256), (unsigned)g.fo);
    ZNN_LAUNCH("direct forward (generic)", s, k_direct_fwd_generic, grid, dim3(256), 0, g, in, w, out);
    return check_launch("direct forward (generic)");
}

int direct_bwd_generic(const Geom& g, const float* gout, const float* w, float* gin, hipStream_t s)
{
    dim3 grid((unsigned)((g.nvol() + 255) / 256), (unsigned)g.f);
    ZNN_LAUNCH("direct backward (generic)", s, k_direct_bwd_generic, grid, dim3(256), 0, g, gout, w, gin);
    return check_launch("direct backward (generic)");
}

int direct_wgrad_generic(const Geom& g, const float* in, const float* gout, float* gw, hipStream_t s)
{
    const long blocks = (long)g.f * g.fo * g.kvol();
    if (blocks >= 2147483647L) return fail(ZNN_EUNSUPPORTED, "too many kernel taps for one launch");
    ZNN_LAUNCH("direct kernel gradient (generic)", s, k_direct_wgrad_generic, dim3((unsigned)blocks), dim3(256), 0, g, in, gout, gw);
    return check_launch("direct kernel gradient (generic)");
}

}  // namespace znn
