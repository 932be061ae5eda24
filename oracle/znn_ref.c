/*
 * znn_ref.c -- CPU oracle for the convolutional-layer hot path of ZNN
 * (arXiv 1510.06706).  TEST INFRASTRUCTURE ONLY: it exists so that the GPU
 * library can be checked against the plain definitions.  It shares no code
 * with the GPU library and must never be called from the product path.
 *
 * Everything is the textbook definition written as nested loops in double
 * precision.  No blocking, no fusion, no FFT.  OpenMP is used only across
 * whole output maps (or whole kernels), the inner loops stay plain.
 *
 * Layouts (row-major, x fastest):
 *   images   [map][z][y][x]
 *   kernels  [fan_out][fan_in][kz][ky][kx]
 *
 * A layer maps f input nodes to f' output nodes through f*f' convolution
 * edges; a node sums the outputs of the edges converging on it
 * (Section 2, "Computation graph").
 *
 * Pins (tests/test_oracle_pins.py): brute-force scatter form on tiny integer
 * inputs, off-centre delta kernels, adjoint identities, finite differences,
 * scipy.signal convolve/correlate, scipy.ndimage.maximum_filter, k = 1 and
 * k = n special cases, fan-in linearity.  No function here is unpinned.
 */
#include <stddef.h>
#include <stdint.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ZNN_REF_OK 0
#define ZNN_REF_EINVAL (-1)

int znn_ref_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Sparse convolution (Section 2): only every s-th voxel of the window enters the sum, so a
 * kernel of k taps spans s*(k-1)+1 voxels and the output extent is n - s*(k-1). */
static int bad_conv(int f, int fo, const int n[3], const int k[3], const int s[3])
{
    if (f < 1 || fo < 1) return 1;
    for (int d = 0; d < 3; ++d)
        if (n[d] < 1 || k[d] < 1 || s[d] < 1 || (long)s[d] * (k[d] - 1) + 1 > n[d]) return 1;
    return 0;
}

/*
 * Forward pass: valid convolution per edge (Section 2, "Convolution"; the
 * footnote there names MATLAB's "valid"), summed over the edges that converge
 * on each output node.  True convolution: the kernel index runs against the
 * image index.
 *
 *   out[j][z][y][x] = sum_i sum_{a,b,c} w[j][i][a][b][c]
 *                       * in[i][z + sz(kz-1-a)][y + sy(ky-1-b)][x + sx(kx-1-c)]
 *
 * (s = sparsity; s = 1 is the dense convolution.)
 */
int znn_ref_conv3d_fwd(int f, int fo, const int n[3], const int k[3], const int s[3],
                       const double *in, const double *w, double *out)
{
    if (bad_conv(f, fo, n, k, s) || !in || !w || !out) return ZNN_REF_EINVAL;
    const int nz = n[0], ny = n[1], nx = n[2];
    const int kz = k[0], ky = k[1], kx = k[2];
    const int sz = s[0], sy = s[1], sx = s[2];
    const int oz = nz - sz * (kz - 1), oy = ny - sy * (ky - 1), ox = nx - sx * (kx - 1);
    const size_t nvol = (size_t)nz * ny * nx, kvol = (size_t)kz * ky * kx;
    const size_t ovol = (size_t)oz * oy * ox;
#pragma omp parallel for schedule(dynamic, 1)
    for (int j = 0; j < fo; ++j) {
        for (int z = 0; z < oz; ++z)
        for (int y = 0; y < oy; ++y)
        for (int x = 0; x < ox; ++x) {
            double acc = 0.0;
            for (int i = 0; i < f; ++i) {
                const double *img = in + (size_t)i * nvol;
                const double *ker = w + ((size_t)j * f + i) * kvol;
                for (int a = 0; a < kz; ++a)
                for (int b = 0; b < ky; ++b)
                for (int c = 0; c < kx; ++c)
                    acc += ker[((size_t)a * ky + b) * kx + c] *
                           img[((size_t)(z + sz * (kz - 1 - a)) * ny + (y + sy * (ky - 1 - b))) * nx +
                               (x + sx * (kx - 1 - c))];
            }
            out[(size_t)j * ovol + ((size_t)z * oy + y) * ox + x] = acc;
        }
    }
    return ZNN_REF_OK;
}

/*
 * Backward pass: the transposed Jacobian of the forward edge is a full
 * convolution with the kernel reflected along all three axes (Section 3.1,
 * "Convolution Jacobian"); an input node sums over its outgoing edges.
 * Reflecting the kernel of a true convolution leaves a correlation:
 *
 *   gin[i][z][y][x] = sum_j sum_{a,b,c} w[j][i][a][b][c]
 *                       * gout[j][z - sz(kz-1-a)][y - sy(ky-1-b)][x - sx(kx-1-c)]
 *
 * where terms whose gout index leaves the image are zero.
 */
int znn_ref_conv3d_bwd(int f, int fo, const int n[3], const int k[3], const int s[3],
                       const double *gout, const double *w, double *gin)
{
    if (bad_conv(f, fo, n, k, s) || !gout || !w || !gin) return ZNN_REF_EINVAL;
    const int nz = n[0], ny = n[1], nx = n[2];
    const int kz = k[0], ky = k[1], kx = k[2];
    const int sz = s[0], sy = s[1], sx = s[2];
    const int oz = nz - sz * (kz - 1), oy = ny - sy * (ky - 1), ox = nx - sx * (kx - 1);
    const size_t nvol = (size_t)nz * ny * nx, kvol = (size_t)kz * ky * kx;
    const size_t ovol = (size_t)oz * oy * ox;
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < f; ++i) {
        for (int z = 0; z < nz; ++z)
        for (int y = 0; y < ny; ++y)
        for (int x = 0; x < nx; ++x) {
            double acc = 0.0;
            for (int j = 0; j < fo; ++j) {
                const double *g = gout + (size_t)j * ovol;
                const double *ker = w + ((size_t)j * f + i) * kvol;
                for (int a = 0; a < kz; ++a) {
                    const int gz = z - sz * (kz - 1 - a);
                    if (gz < 0 || gz >= oz) continue;
                    for (int b = 0; b < ky; ++b) {
                        const int gy = y - sy * (ky - 1 - b);
                        if (gy < 0 || gy >= oy) continue;
                        for (int c = 0; c < kx; ++c) {
                            const int gx = x - sx * (kx - 1 - c);
                            if (gx < 0 || gx >= ox) continue;
                            acc += ker[((size_t)a * ky + b) * kx + c] *
                                   g[((size_t)gz * oy + gy) * ox + gx];
                        }
                    }
                }
            }
            gin[(size_t)i * nvol + ((size_t)z * ny + y) * nx + x] = acc;
        }
    }
    return ZNN_REF_OK;
}

/*
 * Kernel gradient: valid convolution of the reflected forward image at the
 * source node with the backward image at the target node, kernel-sized
 * (Section 3.2, "Kernel update").
 *
 *   gw[j][i][a][b][c] = sum_{z,y,x} gout[j][z][y][x]
 *                         * in[i][z + sz(kz-1-a)][y + sy(ky-1-b)][x + sx(kx-1-c)]
 */
int znn_ref_conv3d_wgrad(int f, int fo, const int n[3], const int k[3], const int s[3],
                         const double *in, const double *gout, double *gw)
{
    if (bad_conv(f, fo, n, k, s) || !in || !gout || !gw) return ZNN_REF_EINVAL;
    const int nz = n[0], ny = n[1], nx = n[2];
    const int kz = k[0], ky = k[1], kx = k[2];
    const int sz = s[0], sy = s[1], sx = s[2];
    const int oz = nz - sz * (kz - 1), oy = ny - sy * (ky - 1), ox = nx - sx * (kx - 1);
    const size_t nvol = (size_t)nz * ny * nx, kvol = (size_t)kz * ky * kx;
    const size_t ovol = (size_t)oz * oy * ox;
    const long pairs = (long)f * fo;
#pragma omp parallel for schedule(dynamic, 1)
    for (long e = 0; e < pairs; ++e) {
        const int j = (int)(e / f), i = (int)(e % f);
        const double *img = in + (size_t)i * nvol;
        const double *g = gout + (size_t)j * ovol;
        for (int a = 0; a < kz; ++a)
        for (int b = 0; b < ky; ++b)
        for (int c = 0; c < kx; ++c) {
            double acc = 0.0;
            for (int z = 0; z < oz; ++z)
            for (int y = 0; y < oy; ++y)
            for (int x = 0; x < ox; ++x)
                acc += g[((size_t)z * oy + y) * ox + x] *
                       img[((size_t)(z + sz * (kz - 1 - a)) * ny + (y + sy * (ky - 1 - b))) * nx +
                           (x + sx * (kx - 1 - c))];
            gw[(size_t)e * kvol + ((size_t)a * ky + b) * kx + c] = acc;
        }
    }
    return ZNN_REF_OK;
}

/*
 * The same three definitions evaluated at chosen output positions only, so a
 * layer too large for a full CPU pass can still be checked element by element.
 * pos[s] is the flat index into the full output tensor of that pass.
 */
int znn_ref_conv3d_fwd_at(int f, int fo, const int n[3], const int k[3], const int s[3],
                          const double *in, const double *w,
                          long count, const int64_t *pos, double *val)
{
    if (bad_conv(f, fo, n, k, s) || !in || !w || !pos || !val || count < 0) return ZNN_REF_EINVAL;
    const int nz = n[0], ny = n[1], nx = n[2];
    const int kz = k[0], ky = k[1], kx = k[2];
    const int sz = s[0], sy = s[1], sx = s[2];
    const int oz = nz - sz * (kz - 1), oy = ny - sy * (ky - 1), ox = nx - sx * (kx - 1);
    const size_t nvol = (size_t)nz * ny * nx, kvol = (size_t)kz * ky * kx;
    const size_t ovol = (size_t)oz * oy * ox;
    for (long s = 0; s < count; ++s)
        if (pos[s] < 0 || (size_t)pos[s] >= ovol * fo) return ZNN_REF_EINVAL;
#pragma omp parallel for schedule(dynamic, 16)
    for (long s = 0; s < count; ++s) {
        size_t p = (size_t)pos[s];
        const int j = (int)(p / ovol); p %= ovol;
        const int z = (int)(p / ((size_t)oy * ox)); p %= (size_t)oy * ox;
        const int y = (int)(p / ox), x = (int)(p % ox);
        double acc = 0.0;
        for (int i = 0; i < f; ++i) {
            const double *img = in + (size_t)i * nvol;
            const double *ker = w + ((size_t)j * f + i) * kvol;
            for (int a = 0; a < kz; ++a)
            for (int b = 0; b < ky; ++b)
            for (int c = 0; c < kx; ++c)
                acc += ker[((size_t)a * ky + b) * kx + c] *
                       img[((size_t)(z + sz * (kz - 1 - a)) * ny + (y + sy * (ky - 1 - b))) * nx +
                           (x + sx * (kx - 1 - c))];
        }
        val[s] = acc;
    }
    return ZNN_REF_OK;
}

int znn_ref_conv3d_bwd_at(int f, int fo, const int n[3], const int k[3], const int s[3],
                          const double *gout, const double *w,
                          long count, const int64_t *pos, double *val)
{
    if (bad_conv(f, fo, n, k, s) || !gout || !w || !pos || !val || count < 0) return ZNN_REF_EINVAL;
    const int nz = n[0], ny = n[1], nx = n[2];
    const int kz = k[0], ky = k[1], kx = k[2];
    const int sz = s[0], sy = s[1], sx = s[2];
    const int oz = nz - sz * (kz - 1), oy = ny - sy * (ky - 1), ox = nx - sx * (kx - 1);
    const size_t nvol = (size_t)nz * ny * nx, kvol = (size_t)kz * ky * kx;
    const size_t ovol = (size_t)oz * oy * ox;
    for (long s = 0; s < count; ++s)
        if (pos[s] < 0 || (size_t)pos[s] >= nvol * f) return ZNN_REF_EINVAL;
#pragma omp parallel for schedule(dynamic, 16)
    for (long s = 0; s < count; ++s) {
        size_t p = (size_t)pos[s];
        const int i = (int)(p / nvol); p %= nvol;
        const int z = (int)(p / ((size_t)ny * nx)); p %= (size_t)ny * nx;
        const int y = (int)(p / nx), x = (int)(p % nx);
        double acc = 0.0;
        for (int j = 0; j < fo; ++j) {
            const double *g = gout + (size_t)j * ovol;
            const double *ker = w + ((size_t)j * f + i) * kvol;
            for (int a = 0; a < kz; ++a) {
                const int gz = z - sz * (kz - 1 - a);
                if (gz < 0 || gz >= oz) continue;
                for (int b = 0; b < ky; ++b) {
                    const int gy = y - sy * (ky - 1 - b);
                    if (gy < 0 || gy >= oy) continue;
                    for (int c = 0; c < kx; ++c) {
                        const int gx = x - sx * (kx - 1 - c);
                        if (gx < 0 || gx >= ox) continue;
                        acc += ker[((size_t)a * ky + b) * kx + c] *
                               g[((size_t)gz * oy + gy) * ox + gx];
                    }
                }
            }
        }
        val[s] = acc;
    }
    return ZNN_REF_OK;
}

int znn_ref_conv3d_wgrad_at(int f, int fo, const int n[3], const int k[3], const int s[3],
                            const double *in, const double *gout,
                            long count, const int64_t *pos, double *val)
{
    if (bad_conv(f, fo, n, k, s) || !in || !gout || !pos || !val || count < 0) return ZNN_REF_EINVAL;
    const int nz = n[0], ny = n[1], nx = n[2];
    const int kz = k[0], ky = k[1], kx = k[2];
    const int sz = s[0], sy = s[1], sx = s[2];
    const int oz = nz - sz * (kz - 1), oy = ny - sy * (ky - 1), ox = nx - sx * (kx - 1);
    const size_t nvol = (size_t)nz * ny * nx, kvol = (size_t)kz * ky * kx;
    const size_t ovol = (size_t)oz * oy * ox;
    for (long s = 0; s < count; ++s)
        if (pos[s] < 0 || (size_t)pos[s] >= kvol * f * fo) return ZNN_REF_EINVAL;
#pragma omp parallel for schedule(dynamic, 4)
    for (long s = 0; s < count; ++s) {
        size_t p = (size_t)pos[s];
        const size_t e = p / kvol; p %= kvol;
        const int j = (int)(e / f), i = (int)(e % f);
        const int a = (int)(p / ((size_t)ky * kx)); p %= (size_t)ky * kx;
        const int b = (int)(p / kx), c = (int)(p % kx);
        const double *img = in + (size_t)i * nvol;
        const double *g = gout + (size_t)j * ovol;
        double acc = 0.0;
        for (int z = 0; z < oz; ++z)
        for (int y = 0; y < oy; ++y)
        for (int x = 0; x < ox; ++x)
            acc += g[((size_t)z * oy + y) * ox + x] *
                   img[((size_t)(z + sz * (kz - 1 - a)) * ny + (y + sy * (ky - 1 - b))) * nx +
                       (x + sx * (kx - 1 - c))];
        val[s] = acc;
    }
    return ZNN_REF_OK;
}

/*
 * Max-filtering (Section 2, "Max-filtering"): the maximum inside a sliding
 * window.  idx records which input voxel supplied the maximum, as the flat
 * offset (z*ny + y)*nx + x inside that map.  The paper does not fix which
 * voxel wins among equal values; this oracle scans the window in ascending
 * flat order with a strict '>' so the smallest flat index wins (-0.0 and +0.0
 * compare equal).
 *
 * The window may be sparse like a convolution's: its win taps lie s voxels
 * apart, and the output extent is n - s (win - 1).  The paper states sparsity
 * for convolutions only; a max-filter that follows an earlier max-filter in a
 * max-filtering ConvNet needs the same treatment for the net to reproduce a
 * sliding-window max-pooling ConvNet (Section 2, last paragraphs, and the
 * figure there), so the filter takes a sparsity too.  s = 1 is the dense filter.
 */
static int bad_filter(int maps, const int n[3], const int win[3], const int s[3])
{
    if (maps < 1) return 1;
    for (int d = 0; d < 3; ++d)
        if (n[d] < 1 || win[d] < 1 || s[d] < 1 || (long)s[d] * (win[d] - 1) + 1 > n[d]) return 1;
    return 0;
}

int znn_ref_maxfilter3d_fwd(int maps, const int n[3], const int win[3], const int s[3],
                            const double *in, double *out, int32_t *idx)
{
    if (!in || !out || !idx || bad_filter(maps, n, win, s)) return ZNN_REF_EINVAL;
    const int nz = n[0], ny = n[1], nx = n[2];
    const int oz = nz - s[0] * (win[0] - 1), oy = ny - s[1] * (win[1] - 1), ox = nx - s[2] * (win[2] - 1);
    const size_t nvol = (size_t)nz * ny * nx, ovol = (size_t)oz * oy * ox;
#pragma omp parallel for schedule(dynamic, 1)
    for (int m = 0; m < maps; ++m) {
        const double *img = in + (size_t)m * nvol;
        for (int z = 0; z < oz; ++z)
        for (int y = 0; y < oy; ++y)
        for (int x = 0; x < ox; ++x) {
            size_t best = ((size_t)z * ny + y) * nx + x;
            double bv = img[best];
            for (int a = 0; a < win[0]; ++a)
            for (int b = 0; b < win[1]; ++b)
            for (int c = 0; c < win[2]; ++c) {
                const size_t q = ((size_t)(z + s[0] * a) * ny + (y + s[1] * b)) * nx + (x + s[2] * c);
                if (img[q] > bv) { bv = img[q]; best = q; }
            }
            const size_t o = (size_t)m * ovol + ((size_t)z * oy + y) * ox + x;
            out[o] = bv;
            idx[o] = (int32_t)best;
        }
    }
    return ZNN_REF_OK;
}

/*
 * Max-filtering Jacobian (Section 3.1): start from a zero image of the
 * filter's input size; for every window position add the incoming value to
 * the voxel that supplied the forward maximum of that window.
 */
int znn_ref_maxfilter3d_bwd(int maps, const int n[3], const int win[3], const int s[3],
                            const double *gout, const int32_t *idx, double *gin)
{
    if (!gout || !idx || !gin || bad_filter(maps, n, win, s)) return ZNN_REF_EINVAL;
    const size_t nvol = (size_t)n[0] * n[1] * n[2];
    const size_t ovol = (size_t)(n[0] - s[0] * (win[0] - 1)) * (n[1] - s[1] * (win[1] - 1)) *
                        (n[2] - s[2] * (win[2] - 1));
    for (size_t p = 0; p < ovol * maps; ++p)
        if (idx[p] < 0 || (size_t)idx[p] >= nvol) return ZNN_REF_EINVAL;
#pragma omp parallel for schedule(dynamic, 1)
    for (int m = 0; m < maps; ++m) {
        double *g = gin + (size_t)m * nvol;
        for (size_t q = 0; q < nvol; ++q) g[q] = 0.0;
        for (size_t p = 0; p < ovol; ++p)
            g[idx[(size_t)m * ovol + p]] += gout[(size_t)m * ovol + p];
    }
    return ZNN_REF_OK;
}

/*
 * Max-pooling (Section 2, "Max-pooling"): the image is cut into blocks of
 * p voxels per axis (n divisible by p) and every block yields its maximum;
 * output extent n / p.  idx is the flat offset inside the input map of the
 * voxel that supplied it; ties go to the smallest flat offset, as above.
 */
int znn_ref_maxpool3d_fwd(int maps, const int n[3], const int p[3],
                          const double *in, double *out, int32_t *idx)
{
    if (maps < 1 || !in || !out || !idx) return ZNN_REF_EINVAL;
    for (int d = 0; d < 3; ++d)
        if (n[d] < 1 || p[d] < 1 || n[d] % p[d] != 0) return ZNN_REF_EINVAL;
    const int ny = n[1], nx = n[2];
    const int oz = n[0] / p[0], oy = n[1] / p[1], ox = n[2] / p[2];
    const size_t nvol = (size_t)n[0] * ny * nx, ovol = (size_t)oz * oy * ox;
#pragma omp parallel for schedule(dynamic, 1)
    for (int m = 0; m < maps; ++m) {
        const double *img = in + (size_t)m * nvol;
        for (int z = 0; z < oz; ++z)
        for (int y = 0; y < oy; ++y)
        for (int x = 0; x < ox; ++x) {
            size_t best = ((size_t)(z * p[0]) * ny + y * p[1]) * nx + x * p[2];
            double bv = img[best];
            for (int a = 0; a < p[0]; ++a)
            for (int b = 0; b < p[1]; ++b)
            for (int c = 0; c < p[2]; ++c) {
                const size_t q = ((size_t)(z * p[0] + a) * ny + (y * p[1] + b)) * nx + (x * p[2] + c);
                if (img[q] > bv) { bv = img[q]; best = q; }
            }
            const size_t o = (size_t)m * ovol + ((size_t)z * oy + y) * ox + x;
            out[o] = bv;
            idx[o] = (int32_t)best;
        }
    }
    return ZNN_REF_OK;
}

/*
 * Max-pooling Jacobian (Section 3.1): the pooled image is expanded back to
 * the input size; inside every block all voxels are zero except the one that
 * was the forward maximum, which receives the block's incoming value.
 */
int znn_ref_maxpool3d_bwd(int maps, const int n[3], const int p[3],
                          const double *gout, const int32_t *idx, double *gin)
{
    if (maps < 1 || !gout || !idx || !gin) return ZNN_REF_EINVAL;
    for (int d = 0; d < 3; ++d)
        if (n[d] < 1 || p[d] < 1 || n[d] % p[d] != 0) return ZNN_REF_EINVAL;
    const size_t nvol = (size_t)n[0] * n[1] * n[2];
    const size_t ovol = (size_t)(n[0] / p[0]) * (n[1] / p[1]) * (n[2] / p[2]);
    for (size_t q = 0; q < ovol * maps; ++q)
        if (idx[q] < 0 || (size_t)idx[q] >= nvol) return ZNN_REF_EINVAL;
    for (int m = 0; m < maps; ++m) {
        double *g = gin + (size_t)m * nvol;
        for (size_t q = 0; q < nvol; ++q) g[q] = 0.0;
        for (size_t q = 0; q < ovol; ++q)
            g[idx[(size_t)m * ovol + q]] = gout[(size_t)m * ovol + q];
    }
    return ZNN_REF_OK;
}
