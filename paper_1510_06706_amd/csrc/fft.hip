// FFT method (Section 4): batched 3D real-to-complex and inverse transforms,
// the per-frequency complex multiply-accumulate that fuses the sum over
// convergent edges, and the pruned inverse transforms of the kernel gradient.
//
// A 3D transform is three launches, one per axis.  The x pass (contiguous
// pencils, two real rows packed into one complex transform) and every pass of
// an extent above 96 stage a batch of W pencils in LDS as data[element][pencil]
// (pencil fastest, row length Wp odd so that the transposing loads and stores
// spread over the banks) and run a Stockham autosort FFT with radices 4/2/3/5
// between two LDS buffers.  The y and z passes of 5-smooth extents up to 96 keep
// one whole pencil per thread in registers instead (fft_reg_impl.h): their
// neighbouring pencils are contiguous in memory, so no transpose is needed.
// Input rows known to be zero (padding) are never read and output rows nobody
// needs (outside the crop) are never written, so the transforms of the small
// kernels and the cropped inverses are pruned for free.
//
// Spectra are stored as [map][N_z][N_y][N_x/2+1] complex fp32.
//
// Fourier-domain identities used (G_s = output gradient embedded at offset k-1
// in the N-volume; any N >= n is free of wrap-around):
//   forward   out = crop_{[k-1, n-1]} IFFT( sum_i W^[j][i] I^[i] )
//   backward  gin = crop_{[0, n)}     IFFT( sum_j conj(W^[j][i]) G_s^[j] )
//   gradient  gw  = crop_{[0, k)}     IFFT( G_s^[j] conj(I^[i]) )
#include "znn_internal.h"

#include <algorithm>
#include <cstdlib>

namespace znn {

namespace {

constexpr int kThreads = 256;

// Radix sequence of a transform; fs[i] divides by the stride s of pass i (the product of
// the radices before it) and fw by the number of pencils per batch, so that the
// butterfly loops decompose their flat index without integer division.
struct Radices { int n; int r[12]; FastDiv fs[12]; FastDiv fw; };

Radices factorize(int N, int W)
{
    Radices R; R.n = 0;
    // long pencils: radix-16 and radix-8 passes (a 16- or 8-point transform in registers per thread) halve
    // the number of trips through LDS and of barriers
    if (N > 96) {
        while (N % 16 == 0) { R.r[R.n++] = 16; N /= 16; }
        if (N % 8 == 0) { R.r[R.n++] = 8; N /= 8; }
    }
    while (N % 4 == 0) { R.r[R.n++] = 4; N /= 4; }
    while (N % 2 == 0) { R.r[R.n++] = 2; N /= 2; }
    while (N % 3 == 0) { R.r[R.n++] = 3; N /= 3; }
    while (N % 5 == 0) { R.r[R.n++] = 5; N /= 5; }
    int s = 1;
    for (int i = 0; i < R.n; ++i) { R.fs[i] = make_fastdiv((unsigned)s); s *= R.r[i]; }
    R.fw = make_fastdiv((unsigned)W);
    return R;
}

// Largest odd pencil-row length such that two N x Wp buffers plus N twiddles fit a workgroup's share of LDS.
// Unless tuned: 24 KiB for the x passes (rows are contiguous, so small batches cost nothing and more
// workgroups per compute unit hide more latency: 256-point r2c 37 -> 25 us against 64 KiB) and 40 KiB for the
// strided passes (whose batches are runs of neighbouring pencils: shorter runs coalesce worse).
int max_row_len(int N, bool x_pass)
{
    const int kb = tuning().fft_lds_kb ? tuning().fft_lds_kb : x_pass ? 24 : 40;
    int lim = (kb * 1024 / 8 - N) / (2 * N);
    if (lim < 1) lim = 1;
    if ((lim & 1) == 0) --lim;
    return lim;
}

size_t lds_bytes(int N, int Wp) { return (size_t)(2 * N * Wp + N) * sizeof(float2); }

__device__ __forceinline__ float2 cadd(float2 a, float2 b) { return make_float2(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ float2 csub(float2 a, float2 b) { return make_float2(a.x - b.x, a.y - b.y); }
__device__ __forceinline__ float2 cmul(float2 a, float2 b)
{
    return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
// multiply by  DIR * i
template <int DIR> __device__ __forceinline__ float2 mul_di(float2 a)
{
    return DIR > 0 ? make_float2(-a.y, a.x) : make_float2(a.y, -a.x);
}

__device__ __forceinline__ void make_twiddles(float2* tw, int N, int dir)
{
    for (int t = threadIdx.x; t < N; t += kThreads) {
        float s, c;
        sincospif(2.0f * (float)t / (float)N, &s, &c);
        tw[t] = make_float2(c, dir > 0 ? s : -s);
    }
}

// 4-point transform in place: b_k = sum_n a_n exp(DIR 2 pi i n k / 4).
template <int DIR>
__device__ __forceinline__ void dft4(float2& a0, float2& a1, float2& a2, float2& a3)
{
    const float2 s02 = cadd(a0, a2), d02 = csub(a0, a2);
    const float2 s13 = cadd(a1, a3), d13 = mul_di<DIR>(csub(a1, a3));
    a0 = cadd(s02, s13);
    a1 = cadd(d02, d13);
    a2 = csub(s02, s13);
    a3 = csub(d02, d13);
}

// a * (c + DIR i s)
template <int DIR> __device__ __forceinline__ float2 cmul_const(float2 a, float c, float s)
{
    return DIR > 0 ? make_float2(a.x * c - a.y * s, a.x * s + a.y * c) : make_float2(a.x * c + a.y * s, a.y * c - a.x * s);
}

// 16-point transform, v[n] -> v[k], as 4 x 4: with n = 4 n1 + n2 and k = k1 + 4 k2,
// exp(2 pi i n k / 16) = w4^(n1 k1) w16^(n2 k1) w4^(n2 k2).
template <int DIR>
__device__ __forceinline__ void dft16(float2 (&v)[16])
{
    constexpr float c1 = 0.9238795325112867f, s1 = 0.3826834323650898f, h = 0.7071067811865476f;
#pragma unroll
    for (int n2 = 0; n2 < 4; ++n2) dft4<DIR>(v[n2], v[n2 + 4], v[n2 + 8], v[n2 + 12]);    // v[n2 + 4 k1]
    // twiddles w16^(n2 k1)
    v[1 + 4] = cmul_const<DIR>(v[1 + 4], c1, s1);
    v[1 + 8] = cmul_const<DIR>(v[1 + 8], h, h);
    v[1 + 12] = cmul_const<DIR>(v[1 + 12], s1, c1);
    v[2 + 4] = cmul_const<DIR>(v[2 + 4], h, h);
    v[2 + 8] = mul_di<DIR>(v[2 + 8]);
    v[2 + 12] = cmul_const<DIR>(v[2 + 12], -h, h);
    v[3 + 4] = cmul_const<DIR>(v[3 + 4], s1, c1);
    v[3 + 8] = cmul_const<DIR>(v[3 + 8], -h, h);
    v[3 + 12] = cmul_const<DIR>(v[3 + 12], -c1, -s1);
#pragma unroll
    for (int k1 = 0; k1 < 4; ++k1) dft4<DIR>(v[4 * k1], v[4 * k1 + 1], v[4 * k1 + 2], v[4 * k1 + 3]);   // v[4 k1 + k2]
    // to natural order k = k1 + 4 k2: transpose the 4 x 4 array
#pragma unroll
    for (int k1 = 0; k1 < 4; ++k1)
#pragma unroll
        for (int k2 = k1 + 1; k2 < 4; ++k2) {
            const float2 t = v[4 * k1 + k2];
            v[4 * k1 + k2] = v[4 * k2 + k1];
            v[4 * k2 + k1] = t;
        }
}

// 8-point transform, v[n] -> v[k], as 4 x 2: with n = 2 n1 + n2 and k = k1 + 4 k2,
// exp(2 pi i n k / 8) = w4^(n1 k1) w8^(n2 k1) (-1)^(n2 k2).
template <int DIR>
__device__ __forceinline__ void dft8(float2 (&v)[8])
{
    constexpr float h = 0.7071067811865476f;
    dft4<DIR>(v[0], v[2], v[4], v[6]);      // n2 = 0: v[2 k1]
    dft4<DIR>(v[1], v[3], v[5], v[7]);      // n2 = 1: v[2 k1 + 1]
    v[3] = cmul_const<DIR>(v[3], h, h);
    v[5] = mul_di<DIR>(v[5]);
    v[7] = cmul_const<DIR>(v[7], -h, h);
    float2 o[8];
#pragma unroll
    for (int k1 = 0; k1 < 4; ++k1) {
        o[k1] = cadd(v[2 * k1], v[2 * k1 + 1]);
        o[k1 + 4] = csub(v[2 * k1], v[2 * k1 + 1]);
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = o[k];
}

// Stockham autosort FFT of W pencils of length N held as src[e * Wp + p].
// DIR = -1: forward kernel exp(-2 pi i jk/N); DIR = +1: unnormalised inverse.
// Returns the buffer that holds the result (natural order).
template <int DIR>
__device__ float2* lds_fft(float2* src, float2* dst, const float2* tw, int N, int W, int Wp,
                           const Radices& R)
{
    int s = 1, n = N;
    for (int ri = 0; ri < R.n; ++ri) {
        const int r = R.r[ri];
        const int m = n / r;
        const int units = m * s * W;
        const int xs = s * m * Wp;   // distance between the r inputs of a butterfly
        const int ys = s * Wp;       // distance between its r outputs
        const FastDiv fs = R.fs[ri];
        for (int u = threadIdx.x; u < units; u += kThreads) {
            const int t = (int)fdiv((unsigned)u, R.fw);
            const int p = u - t * W;
            const int pp = (int)fdiv((unsigned)t, fs);
            const int q = t - pp * s;
            const float2* x = src + (q + s * pp) * Wp + p;
            float2* y = dst + (q + s * r * pp) * Wp + p;
            const int ti = pp * s;   // twiddle index for output 1: exp(DIR 2 pi i pp / n)
            if (r == 16) {
                float2 v[16];
#pragma unroll
                for (int j = 0; j < 16; ++j) v[j] = x[j * xs];
                dft16<DIR>(v);
                y[0] = v[0];
#pragma unroll
                for (int j = 1; j < 16; ++j) y[j * ys] = cmul(v[j], tw[j * ti]);
            } else if (r == 8) {
                float2 v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = x[j * xs];
                dft8<DIR>(v);
                y[0] = v[0];
#pragma unroll
                for (int j = 1; j < 8; ++j) y[j * ys] = cmul(v[j], tw[j * ti]);
            } else if (r == 4) {
                const float2 a0 = x[0], a1 = x[xs], a2 = x[2 * xs], a3 = x[3 * xs];
                const float2 s02 = cadd(a0, a2), d02 = csub(a0, a2);
                const float2 s13 = cadd(a1, a3), d13 = mul_di<DIR>(csub(a1, a3));
                y[0] = cadd(s02, s13);
                y[ys] = cmul(cadd(d02, d13), tw[ti]);
                y[2 * ys] = cmul(csub(s02, s13), tw[2 * ti]);
                y[3 * ys] = cmul(csub(d02, d13), tw[3 * ti]);
            } else if (r == 2) {
                const float2 a0 = x[0], a1 = x[xs];
                y[0] = cadd(a0, a1);
                y[ys] = cmul(csub(a0, a1), tw[ti]);
            } else if (r == 3) {
                const float2 a0 = x[0], a1 = x[xs], a2 = x[2 * xs];
                const float2 t1 = cadd(a1, a2);
                const float2 t2 = make_float2(a0.x - 0.5f * t1.x, a0.y - 0.5f * t1.y);
                float2 t3 = csub(a1, a2);
                t3 = mul_di<DIR>(make_float2(0.8660254037844386f * t3.x, 0.8660254037844386f * t3.y));
                y[0] = cadd(a0, t1);
                y[ys] = cmul(cadd(t2, t3), tw[ti]);
                y[2 * ys] = cmul(csub(t2, t3), tw[2 * ti]);
            } else {   // r == 5
                const float c1 = 0.30901699437494745f, c2 = -0.8090169943749475f;
                const float s1 = 0.9510565162951535f, s2 = 0.5877852522924731f;
                const float2 a0 = x[0], a1 = x[xs], a2 = x[2 * xs], a3 = x[3 * xs], a4 = x[4 * xs];
                const float2 t1 = cadd(a1, a4), t2 = cadd(a2, a3), t3 = csub(a1, a4), t4 = csub(a2, a3);
                const float2 m1 = make_float2(a0.x + c1 * t1.x + c2 * t2.x, a0.y + c1 * t1.y + c2 * t2.y);
                const float2 m2 = make_float2(a0.x + c2 * t1.x + c1 * t2.x, a0.y + c2 * t1.y + c1 * t2.y);
                const float2 n1 = mul_di<DIR>(make_float2(s1 * t3.x + s2 * t4.x, s1 * t3.y + s2 * t4.y));
                const float2 n2 = mul_di<DIR>(make_float2(s2 * t3.x - s1 * t4.x, s2 * t3.y - s1 * t4.y));
                y[0] = cadd(a0, cadd(t1, t2));
                y[ys] = cmul(cadd(m1, n1), tw[ti]);
                y[2 * ys] = cmul(cadd(m2, n2), tw[2 * ti]);
                y[3 * ys] = cmul(csub(m2, n2), tw[3 * ti]);
                y[4 * ys] = cmul(csub(m1, n1), tw[4 * ti]);
            }
        }
        __syncthreads();
        float2* tmp = src; src = dst; dst = tmp;
        n = m;
        s *= r;
    }
    return src;
}

// ---------------------------------------------------------------- x axis, real -> complex
// Source rows are the x-lines of real images [maps][sz][sy][sx]; row (map,z,y)
// lands at spectrum row (map, z+oz, y+oy) with its samples at x+ox of an
// N_x-long zero line.  Two real rows share one complex transform.
struct R2CParams {
    const float* src; float2* dst;
    long rows;
    int sz, sy, sx;
    int Nz, Ny, Nx, Nxh;
    int oz, oy, ox;
    int tz, ty, tx;     // spacing of the source samples inside the volume (1 except for sparse kernels)
    int W, Wp;
    FastDiv fsx, fnxh, fsy, fsz;    // divisions of small block-local numbers by sx, Nxh, sy, sz
    Radices rad;
};

__global__ void __launch_bounds__(kThreads) k_fft_r2c_x(R2CParams P)
{
    extern __shared__ float2 lds[];
    const int N = P.Nx, Wp = P.Wp;
    float2* a = lds;
    float2* b = lds + N * Wp;
    float2* tw = lds + 2 * N * Wp;
    make_twiddles(tw, N, -1);
    for (int t = threadIdx.x; t < N * Wp; t += kThreads) a[t] = make_float2(0.f, 0.f);
    __syncthreads();
    const long row0 = (long)blockIdx.x * (2 * P.W);
    const int nrows = (int)min((long)(2 * P.W), P.rows - row0);
    float* af = reinterpret_cast<float*>(a);
    const float* srow = P.src + row0 * P.sx;
    if (P.tx == 1) {
        for (int t = threadIdx.x; t < nrows * P.sx; t += kThreads) {
            const int r = (int)fdiv((unsigned)t, P.fsx), x = t - r * P.sx;
            af[2 * ((x + P.ox) * Wp + (r >> 1)) + (r & 1)] = srow[t];
        }
    } else {
        for (int t = threadIdx.x; t < nrows * P.sx; t += kThreads) {
            const int r = (int)fdiv((unsigned)t, P.fsx), x = t - r * P.sx;
            af[2 * ((x * P.tx + P.ox) * Wp + (r >> 1)) + (r & 1)] = srow[t];
        }
    }
    __syncthreads();
    const float2* res = lds_fft<-1>(a, b, tw, N, P.W, Wp, P.rad);
    // (map, z, y) of the block's first row: one exact division per block, the rest is
    // block-local and small
    const long map0 = row0 / ((long)P.sy * P.sz);
    const int rem0 = (int)(row0 - map0 * ((long)P.sy * P.sz));
    const int z0 = rem0 / P.sy, y0 = rem0 - z0 * P.sy;
    // split the packed transform: A = (Z[k] + conj Z[N-k]) / 2,  B = (Z[k] - conj Z[N-k]) / (2i)
    for (int t = threadIdx.x; t < nrows * P.Nxh; t += kThreads) {
        const int r = (int)fdiv((unsigned)t, P.fnxh), k = t - r * P.Nxh;
        const int yy = y0 + r;
        const int zc = (int)fdiv((unsigned)yy, P.fsy);
        const int y = yy - zc * P.sy;
        const int zz = z0 + zc;
        const int mc = (int)fdiv((unsigned)zz, P.fsz);
        const int z = zz - mc * P.sz;
        const long map = map0 + mc;
        const float2 z1 = res[k * Wp + (r >> 1)];
        const float2 z2 = res[(k == 0 ? 0 : N - k) * Wp + (r >> 1)];
        float2 v;
        if ((r & 1) == 0) v = make_float2(0.5f * (z1.x + z2.x), 0.5f * (z1.y - z2.y));
        else              v = make_float2(0.5f * (z1.y + z2.y), 0.5f * (z2.x - z1.x));
        P.dst[((map * P.Nz + z * P.tz + P.oz) * P.Ny + (y * P.ty + P.oy)) * P.Nxh + k] = v;
    }
}

// ---------------------------------------------------------------- x axis, complex -> real
// Rows (map, z+cz, y+cy) of a Hermitian half-spectrum become real lines; only
// samples x in [cx, cx+dx) are written, scaled.  Two rows share one transform.
struct C2RParams {
    const float2* src; float* dst;
    long rows;                  // maps * dz * dy
    int cz, cy, cx;
    int dz, dy, dx;
    int Nz, Ny, Nx, Nxh;
    float scale;
    int tx;             // spacing of the wanted samples along x (1 except for sparse kernel gradients)
    int W, Wp;
    FastDiv fdx, fnxh, fdy, fdz;
    Radices rad;
};

__global__ void __launch_bounds__(kThreads) k_fft_c2r_x(C2RParams P)
{
    extern __shared__ float2 lds[];
    const int N = P.Nx, Wp = P.Wp;
    float2* a = lds;
    float2* b = lds + N * Wp;
    float2* tw = lds + 2 * N * Wp;
    make_twiddles(tw, N, +1);
    const long row0 = (long)blockIdx.x * (2 * P.W);
    const int nrows = (int)min((long)(2 * P.W), P.rows - row0);
    const int npen = (nrows + 1) >> 1;
    const long map0 = row0 / ((long)P.dy * P.dz);
    const int rem0 = (int)(row0 - map0 * ((long)P.dy * P.dz));
    const int z0 = rem0 / P.dy, y0 = rem0 - z0 * P.dy;
    for (int t = threadIdx.x; t < npen * P.Nxh; t += kThreads) {
        const int p = (int)fdiv((unsigned)t, P.fnxh), k = t - p * P.Nxh;
        float2 A, B = make_float2(0.f, 0.f);
        {
            const int yy = y0 + 2 * p;
            const int zc = (int)fdiv((unsigned)yy, P.fdy);
            const int y = yy - zc * P.dy;
            const int zz = z0 + zc;
            const int mc = (int)fdiv((unsigned)zz, P.fdz);
            const int z = zz - mc * P.dz;
            A = P.src[(((map0 + mc) * P.Nz + z + P.cz) * P.Ny + (y + P.cy)) * P.Nxh + k];
        }
        if (2 * p + 1 < nrows) {
            const int yy = y0 + 2 * p + 1;
            const int zc = (int)fdiv((unsigned)yy, P.fdy);
            const int y = yy - zc * P.dy;
            const int zz = z0 + zc;
            const int mc = (int)fdiv((unsigned)zz, P.fdz);
            const int z = zz - mc * P.dz;
            B = P.src[(((map0 + mc) * P.Nz + z + P.cz) * P.Ny + (y + P.cy)) * P.Nxh + k];
        }
        // Z = A + iB on the stored half, Hermitian extension on the rest; the
        // imaginary parts of the DC and Nyquist bins of a real line are zero.
        if (k == 0 || 2 * k == N) {
            a[k * Wp + p] = make_float2(A.x, B.x);
        } else {
            a[k * Wp + p] = make_float2(A.x - B.y, A.y + B.x);
            a[(N - k) * Wp + p] = make_float2(A.x + B.y, B.x - A.y);
        }
    }
    __syncthreads();
    const float2* res = lds_fft<+1>(a, b, tw, N, P.W, Wp, P.rad);
    const float* rf = reinterpret_cast<const float*>(res);
    float* drow = P.dst + row0 * P.dx;
    for (int t = threadIdx.x; t < nrows * P.dx; t += kThreads) {
        const int r = (int)fdiv((unsigned)t, P.fdx), x = t - r * P.dx;
        drow[t] = P.scale * rf[2 * ((x * P.tx + P.cx) * Wp + (r >> 1)) + (r & 1)];
    }
}

// ---------------------------------------------------------------- strided axis, complex -> complex
// Pencils run along an axis with element stride `in_stride`; L neighbouring
// pencils are contiguous in memory and are cut into chunks of W.  Three outer
// indices (counts Oa, Ob, Oc) enumerate the remaining dimensions.  Only input
// elements [i0, i0+ni) are read (the rest are zero) and only output elements
// [o0, o0+no) are written, at out + e * out_stride.  With `in2` set the input
// is the product in[...] * conj(in2[...]) (kernel gradient).
struct AxisParams {
    const float2* in; const float2* in2; float2* out;
    int N, i0, ni, o0, no;
    int istep, ostep;   // element e of the input sits at i0 + e*istep; output e is element o0 + e*ostep
    long in_stride, out_stride;
    int L, W, Wp, chunks;
    int Oa, Ob, Oc;
    long in_sa, in_sb, in_sc;
    long in2_sa, in2_sb, in2_sc;
    long out_sa, out_sb, out_sc;
    FastDiv fchunks, foc, fob;      // block index -> (chunk, oc, ob, oa)
    Radices rad;                    // rad.fw divides by W
};

template <int DIR, bool PRODUCT>
__global__ void __launch_bounds__(kThreads) k_fft_axis(AxisParams P)
{
    extern __shared__ float2 lds[];
    const int N = P.N, Wp = P.Wp;
    float2* a = lds;
    float2* b = lds + N * Wp;
    float2* tw = lds + 2 * N * Wp;
    make_twiddles(tw, N, DIR);
    // the launcher keeps the grid below 2^31 / (largest divisor), so these are exact
    const unsigned blk = blockIdx.x;
    unsigned o = fdiv(blk, P.fchunks);
    const int chunk = (int)(blk - o * P.chunks);
    const unsigned o2 = fdiv(o, P.foc);
    const int oc = (int)(o - o2 * P.Oc);
    const int oa = (int)fdiv(o2, P.fob);
    const int ob = (int)(o2 - (unsigned)oa * P.Ob);
    const int p0 = chunk * P.W;
    const int w = min(P.W, P.L - p0);
    if (P.ni < N || P.istep > 1) {
        for (int t = threadIdx.x; t < N * Wp; t += kThreads) a[t] = make_float2(0.f, 0.f);
        __syncthreads();
    }
    const float2* in = P.in + (oa * P.in_sa + ob * P.in_sb + oc * P.in_sc) + p0;
    const float2* in2 = PRODUCT ? P.in2 + (oa * P.in2_sa + ob * P.in2_sb + oc * P.in2_sc) + p0 : nullptr;
    // rows of w pencils; the ragged last chunk (w < W) pays for a real division
    const bool full = w == P.W;
    for (int t = threadIdx.x; t < P.ni * w; t += kThreads) {
        const int row = full ? (int)fdiv((unsigned)t, P.rad.fw) : t / w;
        const int e = row * P.istep + P.i0, p = t - row * w;
        float2 v = in[e * P.in_stride + p];
        if (PRODUCT) {
            const float2 c = in2[e * P.in_stride + p];
            v = make_float2(v.x * c.x + v.y * c.y, v.y * c.x - v.x * c.y);   // v * conj(c)
        }
        a[e * Wp + p] = v;
    }
    __syncthreads();
    const float2* res = lds_fft<DIR>(a, b, tw, N, P.W, Wp, P.rad);
    float2* out = P.out + (oa * P.out_sa + ob * P.out_sb + oc * P.out_sc) + p0;
    for (int t = threadIdx.x; t < P.no * w; t += kThreads) {
        const int q = full ? (int)fdiv((unsigned)t, P.rad.fw) : t / w;
        const int p = t - q * w;
        out[(q + P.o0) * P.out_stride + p] = res[(q * P.ostep + P.o0) * Wp + p];
    }
}

// ---------------------------------------------------------------- per-frequency multiply-accumulate
// Forward:  O^[j][w]  = sum_i W^[j][i][w] I^[i][w]
// Backward: Gin^[i][w] = sum_j conj(W^[j][i][w]) G^[j][w]
// This is the sum over the edges converging on a node, done in the frequency domain.
// A thread owns V neighbouring frequencies and kMacGroup result nodes; it walks the
// reduction index, so the kernel spectra are streamed from HBM exactly once (they are
// not reused: non-temporal loads) while the node spectra stay cache resident.
constexpr int kMacGroup = 8;

typedef float native2 __attribute__((ext_vector_type(2)));
typedef float native4 __attribute__((ext_vector_type(4)));
template <int V> struct CVec;
template <> struct CVec<1> { typedef native2 type; };
template <> struct CVec<2> { typedef native4 type; };

template <bool BWD, int V>
__global__ void __launch_bounds__(kThreads)
k_mac(int f, int fo, long svol, const float2* __restrict__ What, const float2* __restrict__ X,
      float2* __restrict__ Y)
{
    typedef typename CVec<V>::type vec_t;
    const long wv = ((long)blockIdx.x * kThreads + threadIdx.x) * V;
    if (wv >= svol) return;
    const int o0 = blockIdx.y * kMacGroup;
    const int nred = BWD ? fo : f, nout = BWD ? f : fo;
    float acc[kMacGroup][2 * V];
#pragma unroll
    for (int g = 0; g < kMacGroup; ++g)
#pragma unroll
        for (int c = 0; c < 2 * V; ++c) acc[g][c] = 0.f;
#pragma unroll 2
    for (int r = 0; r < nred; ++r) {
        const vec_t xv = *reinterpret_cast<const vec_t*>(X + r * svol + wv);
        const float* x = reinterpret_cast<const float*>(&xv);
#pragma unroll
        for (int g = 0; g < kMacGroup; ++g) {
            if (o0 + g < nout) {
                const long e = BWD ? ((long)r * f + (o0 + g)) : ((long)(o0 + g) * f + r);
                const vec_t kv = __builtin_nontemporal_load(reinterpret_cast<const vec_t*>(What + e * svol + wv));
                const float* k = reinterpret_cast<const float*>(&kv);
#pragma unroll
                for (int c = 0; c < V; ++c) {
                    const float kr = k[2 * c], ki = BWD ? -k[2 * c + 1] : k[2 * c + 1];
                    acc[g][2 * c] = fmaf(kr, x[2 * c], fmaf(-ki, x[2 * c + 1], acc[g][2 * c]));
                    acc[g][2 * c + 1] = fmaf(kr, x[2 * c + 1], fmaf(ki, x[2 * c], acc[g][2 * c + 1]));
                }
            }
        }
    }
#pragma unroll
    for (int g = 0; g < kMacGroup; ++g)
        if (o0 + g < nout) {
            vec_t o;
            float* op = reinterpret_cast<float*>(&o);
#pragma unroll
            for (int c = 0; c < 2 * V; ++c) op[c] = acc[g][c];
            *reinterpret_cast<vec_t*>(Y + (long)(o0 + g) * svol + wv) = o;
        }
}

// ---------------------------------------------------------------- pruned DFTs along z
// When only KZ <= 8 of the N_z input planes are non-zero (kernels) or only KZ output
// planes are wanted (kernel gradient), the z transform is KZ complex multiply-adds per
// element: cheaper than an LDS round trip.  One thread owns a (y, x-frequency) pencil,
// neighbouring threads own neighbouring pencils (coalesced), twiddles are wave-uniform.
constexpr int kMaxPruned = 16;

template <int KZ>
__global__ void __launch_bounds__(kThreads)
k_zdft_expand(float2* __restrict__ spec, int N, int oz, int tz, long plane, long vol, int cpm)
{
    __shared__ float2 tw[kMaxFftExtent];
    make_twiddles(tw, N, -1);
    __syncthreads();
    const long map = blockIdx.x / cpm;
    const long p = (long)(blockIdx.x % cpm) * kThreads + threadIdx.x;
    if (p >= plane) return;
    float2* base = spec + map * vol + p;
    float2 v[KZ];
    int idx[KZ], step[KZ];
#pragma unroll
    for (int a = 0; a < KZ; ++a) {
        v[a] = base[(long)(oz + a * tz) * plane];
        idx[a] = 0;
        step[a] = (oz + a * tz) % N;
    }
    for (int wz = 0; wz < N; ++wz) {
        float2 o = make_float2(0.f, 0.f);
#pragma unroll
        for (int a = 0; a < KZ; ++a) {
            const float2 t = tw[idx[a]];
            o.x = fmaf(v[a].x, t.x, fmaf(-v[a].y, t.y, o.x));
            o.y = fmaf(v[a].x, t.y, fmaf(v[a].y, t.x, o.y));
            idx[a] += step[a];
            if (idx[a] >= N) idx[a] -= N;
        }
        base[(long)wz * plane] = o;
    }
}

// Grid order of the pruned DFTs of the spectral products.  A workgroup owns a block of (j, i)
// pairs and a chunk of 256 pencils; workgroups with the same chunk and the same j block read the
// same output-gradient spectra, those with the same i block the same image spectra.  Consecutive
// workgroups are dealt to the eight XCDs (each with its own L2) in turn, so the flat index is
// taken apart as xcd = b % 8, slot = b / 8, and super-tiles of kTileJ x kTileI pair blocks of one
// pencil chunk are kept on one XCD, next to each other in time: the spectra of a super-tile are
// fetched from HBM once instead of once per workgroup (config 5: 22 GB per launch before, where
// the two node sets hold 0.9 GB).
constexpr int kTileJ = 16, kTileI = 4;
__device__ __forceinline__ bool pair_block_of(unsigned b, int jblocks, int iblocks, int& jblk, int& iblk, int& pchunk)
{
    const int xcd = b & 7, slot = b >> 3;
    const int st = (slot / (kTileJ * kTileI)) * 8 + xcd, within = slot % (kTileJ * kTileI);
    const int sj = (jblocks + kTileJ - 1) / kTileJ, si = (iblocks + kTileI - 1) / kTileI;
    const int ti = st % si, tj = (st / si) % sj;
    pchunk = st / (si * sj);
    jblk = tj * kTileJ + within / kTileI;
    iblk = ti * kTileI + within % kTileI;
    return jblk < jblocks && iblk < iblocks;
}

// T1[j][i][a][p] = sum_z G[j][z][p] conj(I[i][z][p]) exp(+2 pi i a z / N),  a < KZ,
// along the axis whose elements are `plane` apart (z in 3D; y when N_z = 1).
// A thread keeps the sums of a JB x IB block of (j, i) pairs, so every spectrum element
// it loads is used in several products.  Workgroups that share a pencil chunk are
// neighbours in the grid (pair blocks vary fastest), so they find the chunk in cache.
template <int KZ, int JB, int IB>
__global__ void __launch_bounds__(kThreads)
k_wgrad_zdft(const float2* __restrict__ G, const float2* __restrict__ I, float2* __restrict__ T1,
             int f, int fo, int N, int tz, long plane, long vol, int iblocks, int flat)
{
    __shared__ float2 tw[kMaxFftExtent];
    make_twiddles(tw, N, +1);
    __syncthreads();
    int jblk, iblk;
    long p;
    if (flat) {
        // small planes: (pair block, pencil) as one flat index, so that every wave is full
        const long t = (long)blockIdx.x * kThreads + threadIdx.x;
        const long pb = t / plane;
        p = t - pb * plane;
        iblk = (int)(pb % iblocks);
        jblk = (int)(pb / iblocks);
        if (jblk >= (fo + JB - 1) / JB) return;
    } else {
        int pchunk;
        if (!pair_block_of(blockIdx.x, (fo + JB - 1) / JB, iblocks, jblk, iblk, pchunk)) return;
        p = (long)pchunk * kThreads + threadIdx.x;
        if (p >= plane) return;
    }
    const int j0 = jblk * JB, i0 = iblk * IB;
    const float2* gp[JB];
    const float2* ip[IB];
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) gp[jb] = G + (long)min(j0 + jb, fo - 1) * vol + p;
#pragma unroll
    for (int ib = 0; ib < IB; ++ib) ip[ib] = I + (long)min(i0 + ib, f - 1) * vol + p;
    float2 acc[JB][IB][KZ];
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
#pragma unroll
        for (int ib = 0; ib < IB; ++ib)
#pragma unroll
            for (int a = 0; a < KZ; ++a) acc[jb][ib][a] = make_float2(0.f, 0.f);
    int idx[KZ];
#pragma unroll
    for (int a = 0; a < KZ; ++a) idx[a] = 0;
#pragma unroll 2
    for (int z = 0; z < N; ++z) {
        float2 gv[JB], xv[IB], t[KZ];
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) gv[jb] = gp[jb][(long)z * plane];
#pragma unroll
        for (int ib = 0; ib < IB; ++ib) xv[ib] = ip[ib][(long)z * plane];
#pragma unroll
        for (int a = 0; a < KZ; ++a) {
            t[a] = tw[idx[a]];
            idx[a] += a * tz;               // lag a*tz < N
            if (idx[a] >= N) idx[a] -= N;
        }
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
#pragma unroll
            for (int ib = 0; ib < IB; ++ib) {
                // g * conj(x)
                const float pr = fmaf(gv[jb].x, xv[ib].x, gv[jb].y * xv[ib].y);
                const float pi = fmaf(gv[jb].y, xv[ib].x, -gv[jb].x * xv[ib].y);
#pragma unroll
                for (int a = 0; a < KZ; ++a) {
                    acc[jb][ib][a].x = fmaf(pr, t[a].x, fmaf(-pi, t[a].y, acc[jb][ib][a].x));
                    acc[jb][ib][a].y = fmaf(pr, t[a].y, fmaf(pi, t[a].x, acc[jb][ib][a].y));
                }
            }
    }
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
#pragma unroll
        for (int ib = 0; ib < IB; ++ib) {
            const int j = j0 + jb, i = i0 + ib;
            if (j < fo && i < f) {
#pragma unroll
                for (int a = 0; a < KZ; ++a) T1[(((long)j * f + i) * KZ + a) * plane + p] = acc[jb][ib][a];
            }
        }
}

typedef float floatx2 __attribute__((ext_vector_type(2)));
// fourth word of a buffer resource descriptor for untyped loads (32-bit data format, no swizzle)
constexpr int kBufferWord3 = 0x00020000;

// The same sums for N divisible by 4 and lags one voxel apart, four z a quarter period apart at
// a time: with z = z0 + q N/4,
//   T1[a] = sum_z0 exp(+2 pi i a z0 / N) * sum_q prod[z0 + q N/4] i^(a q),
// so the four products are first combined by a radix-4 butterfly of additions into the four
// classes a mod 4, and each lag then costs one complex multiply-add per FOUR z instead of one
// per z (KZ + 1 -> KZ/4 + 2 complex operations per product).
// (FLAT is a template parameter because the pair block of a thread is uniform over the workgroup only
// without it, and only then do the loads get scalar bases.)
template <int KZ, int JB, int IB, bool FLAT>
__global__ void __launch_bounds__(kThreads)
k_wgrad_zdft4(const float2* __restrict__ G, const float2* __restrict__ I, float2* __restrict__ T1,
              int f, int fo, int N, long plane, long vol, int iblocks)
{
    __shared__ float2 tw[kMaxFftExtent];
    make_twiddles(tw, N, +1);
    __syncthreads();
    int jblk, iblk;
    long p;
    if (FLAT) {
        // small planes: (pair block, pencil) as one flat index, so that every wave is full
        const long t = (long)blockIdx.x * kThreads + threadIdx.x;
        const long pb = t / plane;
        p = t - pb * plane;
        iblk = (int)(pb % iblocks);
        jblk = (int)(pb / iblocks);
        if (jblk >= (fo + JB - 1) / JB) return;
    } else {
        int pchunk;
        if (!pair_block_of(blockIdx.x, (fo + JB - 1) / JB, iblocks, jblk, iblk, pchunk)) return;
        p = (long)pchunk * kThreads + threadIdx.x;
        if (p >= plane) return;
    }
    const int j0 = jblk * JB, i0 = iblk * IB;
    const int Q = N >> 2;
    // Spectrum element (map, z, p) = base of the map + z * plane + the thread's p.  Where the maps are uniform
    // over the workgroup (not FLAT) the loads are buffer loads: the map's base in a resource descriptor, the row
    // z * plane * 8 as a scalar offset, p * 8 as the lane's 32-bit offset (the host checks that a map's spectrum
    // stays below 4 GB), which costs no vector instruction; formed as 64-bit pointers per thread the addresses
    // cost 30 vector additions per round of the loop, 6 % of its instructions.
    const float2* gp[JB];
    const float2* ip[IB];
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) gp[jb] = G + (long)min(j0 + jb, fo - 1) * vol;
#pragma unroll
    for (int ib = 0; ib < IB; ++ib) ip[ib] = I + (long)min(i0 + ib, f - 1) * vol;
    __amdgpu_buffer_rsrc_t gr[JB], ir[IB];
    if constexpr (!FLAT) {
        const int bytes = (int)(unsigned)(vol * 8);
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) gr[jb] = __builtin_amdgcn_make_buffer_rsrc((void*)gp[jb], 0, bytes, kBufferWord3);
#pragma unroll
        for (int ib = 0; ib < IB; ++ib) ir[ib] = __builtin_amdgcn_make_buffer_rsrc((void*)ip[ib], 0, bytes, kBufferWord3);
    }
    const int pbytes = (int)((unsigned)p * 8u);
    const unsigned zstep = (unsigned)(plane * 8);
    float2 acc[JB][IB][KZ];
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
#pragma unroll
        for (int ib = 0; ib < IB; ++ib)
#pragma unroll
            for (int a = 0; a < KZ; ++a) acc[jb][ib][a] = make_float2(0.f, 0.f);
    for (int z0 = 0; z0 < Q; ++z0) {
        float2 gv[JB][4], xv[IB][4], t[KZ];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if constexpr (FLAT) {
#pragma unroll
                for (int jb = 0; jb < JB; ++jb) gv[jb][q] = gp[jb][(long)(z0 + q * Q) * plane + p];
#pragma unroll
                for (int ib = 0; ib < IB; ++ib) xv[ib][q] = ip[ib][(long)(z0 + q * Q) * plane + p];
            } else {
                const int zoff = (int)((unsigned)(z0 + q * Q) * zstep);     // uniform
#pragma unroll
                for (int jb = 0; jb < JB; ++jb) {
                    const floatx2 v = __builtin_amdgcn_raw_buffer_load_b64(gr[jb], pbytes, zoff, 0);
                    gv[jb][q] = make_float2(v.x, v.y);
                }
#pragma unroll
                for (int ib = 0; ib < IB; ++ib) {
                    const floatx2 v = __builtin_amdgcn_raw_buffer_load_b64(ir[ib], pbytes, zoff, 0);
                    xv[ib][q] = make_float2(v.x, v.y);
                }
            }
        }
#pragma unroll
        for (int a = 1; a < KZ; ++a) t[a] = tw[(a * z0) % N];       // wave-uniform LDS reads
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
#pragma unroll
            for (int ib = 0; ib < IB; ++ib) {
                float2 pr[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {       // g * conj(x)
                    pr[q].x = fmaf(gv[jb][q].x, xv[ib][q].x, gv[jb][q].y * xv[ib][q].y);
                    pr[q].y = fmaf(gv[jb][q].y, xv[ib][q].x, -gv[jb][q].x * xv[ib][q].y);
                }
                // u[c] = sum_q pr[q] i^(c q)
                const float2 s02 = make_float2(pr[0].x + pr[2].x, pr[0].y + pr[2].y);
                const float2 d02 = make_float2(pr[0].x - pr[2].x, pr[0].y - pr[2].y);
                const float2 s13 = make_float2(pr[1].x + pr[3].x, pr[1].y + pr[3].y);
                const float2 d13 = make_float2(pr[1].x - pr[3].x, pr[1].y - pr[3].y);
                float2 u[4];
                u[0] = make_float2(s02.x + s13.x, s02.y + s13.y);
                u[2] = make_float2(s02.x - s13.x, s02.y - s13.y);
                u[1] = make_float2(d02.x - d13.y, d02.y + d13.x);      // d02 + i d13
                u[3] = make_float2(d02.x + d13.y, d02.y - d13.x);      // d02 - i d13
                acc[jb][ib][0].x += u[0].x;
                acc[jb][ib][0].y += u[0].y;
#pragma unroll
                for (int a = 1; a < KZ; ++a) {
                    const float2 v = u[a & 3];
                    acc[jb][ib][a].x = fmaf(v.x, t[a].x, fmaf(-v.y, t[a].y, acc[jb][ib][a].x));
                    acc[jb][ib][a].y = fmaf(v.x, t[a].y, fmaf(v.y, t[a].x, acc[jb][ib][a].y));
                }
            }
    }
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
#pragma unroll
        for (int ib = 0; ib < IB; ++ib) {
            const int j = j0 + jb, i = i0 + ib;
            if (j < fo && i < f) {
#pragma unroll
                for (int a = 0; a < KZ; ++a) T1[(((long)j * f + i) * KZ + a) * plane + p] = acc[jb][ib][a];
            }
        }
}

// Pruned inverse DFT along an axis of length N whose elements are L apart, for data that is
// already small in every other respect (second axis of the kernel gradient):
//   out[o][b][l] = sum_n in[o][n][l] exp(+2 pi i b t n / N),   b < KY.
// One thread per (o, l); with N divisible by 4 and t = 1 four n a quarter period apart share
// one radix-4 butterfly, as above.  Memory-bound: every input element is read once.
template <int KY>
__global__ void __launch_bounds__(kThreads)
k_prune_idft(const float2* __restrict__ in, float2* __restrict__ out, long outer, int N, int L, int t, int grouped)
{
    __shared__ float2 tw[kMaxFftExtent];
    make_twiddles(tw, N, +1);
    __syncthreads();
    const long id = (long)blockIdx.x * kThreads + threadIdx.x;
    if (id >= outer * L) return;
    const long o = id / L;
    const int l = (int)(id - o * L);
    const float2* src = in + o * (long)N * L + l;
    float2 acc[KY];
#pragma unroll
    for (int b = 0; b < KY; ++b) acc[b] = make_float2(0.f, 0.f);
    if (grouped) {
        const int Q = N >> 2;
        for (int n0 = 0; n0 < Q; ++n0) {
            float2 v[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = src[(long)(n0 + q * Q) * L];
            const float2 s02 = make_float2(v[0].x + v[2].x, v[0].y + v[2].y);
            const float2 d02 = make_float2(v[0].x - v[2].x, v[0].y - v[2].y);
            const float2 s13 = make_float2(v[1].x + v[3].x, v[1].y + v[3].y);
            const float2 d13 = make_float2(v[1].x - v[3].x, v[1].y - v[3].y);
            float2 u[4];
            u[0] = make_float2(s02.x + s13.x, s02.y + s13.y);
            u[2] = make_float2(s02.x - s13.x, s02.y - s13.y);
            u[1] = make_float2(d02.x - d13.y, d02.y + d13.x);
            u[3] = make_float2(d02.x + d13.y, d02.y - d13.x);
            acc[0].x += u[0].x;
            acc[0].y += u[0].y;
#pragma unroll
            for (int b = 1; b < KY; ++b) {
                const float2 w = tw[(b * n0) % N];
                const float2 x = u[b & 3];
                acc[b].x = fmaf(x.x, w.x, fmaf(-x.y, w.y, acc[b].x));
                acc[b].y = fmaf(x.x, w.y, fmaf(x.y, w.x, acc[b].y));
            }
        }
    } else {
        int idx[KY];
#pragma unroll
        for (int b = 0; b < KY; ++b) idx[b] = 0;
        for (int n = 0; n < N; ++n) {
            const float2 x = src[(long)n * L];
#pragma unroll
            for (int b = 0; b < KY; ++b) {
                const float2 w = tw[idx[b]];
                acc[b].x = fmaf(x.x, w.x, fmaf(-x.y, w.y, acc[b].x));
                acc[b].y = fmaf(x.x, w.y, fmaf(x.y, w.x, acc[b].y));
                idx[b] += b * t;            // lag b*t < N
                if (idx[b] >= N) idx[b] -= N;
            }
        }
    }
    float2* dst = out + o * (long)KY * L + l;
#pragma unroll
    for (int b = 0; b < KY; ++b) dst[(long)b * L] = acc[b];
}

template <int KY>
int launch_prune_k(const float2* in, float2* out, long outer, int N, int L, int t, hipStream_t s)
{
    const long blocks = (outer * L + kThreads - 1) / kThreads;
    if (blocks >= 2147483647L) return fail(ZNN_EUNSUPPORTED, "too many pencils for one launch");
    ZNN_LAUNCH("pruned DFT, second axis of the kernel gradient", s, k_prune_idft<KY>, dim3((unsigned)blocks),
               dim3(kThreads), 0, in, out, outer, N, L, t, (N % 4 == 0 && t == 1) ? 1 : 0);
    return check_launch("pruned DFT");
}

int launch_prune(int ky, const float2* in, float2* out, long outer, int N, int L, int t, hipStream_t s)
{
    switch (ky) {
        case 1: return launch_prune_k<1>(in, out, outer, N, L, t, s);
        case 2: return launch_prune_k<2>(in, out, outer, N, L, t, s);
        case 3: return launch_prune_k<3>(in, out, outer, N, L, t, s);
        case 4: return launch_prune_k<4>(in, out, outer, N, L, t, s);
        case 5: return launch_prune_k<5>(in, out, outer, N, L, t, s);
        case 6: return launch_prune_k<6>(in, out, outer, N, L, t, s);
        case 7: return launch_prune_k<7>(in, out, outer, N, L, t, s);
        case 8: return launch_prune_k<8>(in, out, outer, N, L, t, s);
        case 9: return launch_prune_k<9>(in, out, outer, N, L, t, s);
        case 10: return launch_prune_k<10>(in, out, outer, N, L, t, s);
        case 11: return launch_prune_k<11>(in, out, outer, N, L, t, s);
        case 12: return launch_prune_k<12>(in, out, outer, N, L, t, s);
        case 13: return launch_prune_k<13>(in, out, outer, N, L, t, s);
        case 14: return launch_prune_k<14>(in, out, outer, N, L, t, s);
        case 15: return launch_prune_k<15>(in, out, outer, N, L, t, s);
        default: return launch_prune_k<16>(in, out, outer, N, L, t, s);
    }
}

template <int KZ>
int launch_expand_kz(float2* spec, long maps, int N, int oz, int tz, long plane, long vol, hipStream_t s)
{
    const int cpm = (int)((plane + kThreads - 1) / kThreads);
    const long blocks = maps * cpm;
    if (blocks >= 2147483647L) return fail(ZNN_EUNSUPPORTED, "too many pencils for one launch");
    ZNN_LAUNCH("pruned z DFT of kernels", s, k_zdft_expand<KZ>, dim3((unsigned)blocks), dim3(kThreads), 0,
               spec, N, oz, tz, plane, vol, cpm);
    return check_launch("pruned z DFT of kernels");
}

int launch_expand(int kz, float2* spec, long maps, int N, int oz, int tz, long plane, long vol, hipStream_t s)
{
    switch (kz) {
        case 1: return launch_expand_kz<1>(spec, maps, N, oz, tz, plane, vol, s);
        case 2: return launch_expand_kz<2>(spec, maps, N, oz, tz, plane, vol, s);
        case 3: return launch_expand_kz<3>(spec, maps, N, oz, tz, plane, vol, s);
        case 4: return launch_expand_kz<4>(spec, maps, N, oz, tz, plane, vol, s);
        case 5: return launch_expand_kz<5>(spec, maps, N, oz, tz, plane, vol, s);
        case 6: return launch_expand_kz<6>(spec, maps, N, oz, tz, plane, vol, s);
        case 7: return launch_expand_kz<7>(spec, maps, N, oz, tz, plane, vol, s);
        case 8: return launch_expand_kz<8>(spec, maps, N, oz, tz, plane, vol, s);
        case 9: return launch_expand_kz<9>(spec, maps, N, oz, tz, plane, vol, s);
        case 10: return launch_expand_kz<10>(spec, maps, N, oz, tz, plane, vol, s);
        case 11: return launch_expand_kz<11>(spec, maps, N, oz, tz, plane, vol, s);
        case 12: return launch_expand_kz<12>(spec, maps, N, oz, tz, plane, vol, s);
        case 13: return launch_expand_kz<13>(spec, maps, N, oz, tz, plane, vol, s);
        case 14: return launch_expand_kz<14>(spec, maps, N, oz, tz, plane, vol, s);
        case 15: return launch_expand_kz<15>(spec, maps, N, oz, tz, plane, vol, s);
        default: return launch_expand_kz<16>(spec, maps, N, oz, tz, plane, vol, s);
    }
}

// Pruned inverse DFT of the spectral products along the axis with element stride `plane`.
template <int KZ>
int launch_wgrad_dft_k(int f, int fo, int N, int tz, long plane, long vol, const float2* G, const float2* I, float2* T,
                       hipStream_t s)
{
    // pairs per thread: as many as the register file takes next to their 2 KZ sums each (config 5, KZ = 7:
    // 2 x 4 pairs 3.57 ms, 3 x 3 pairs 3.18 ms: fewer loads per pair; the 2D benchmark layer, KZ = 11, whose planes
    // give few threads, is faster with 2 x 2 than with 2 x 3: 0.29 against 0.37 ms)
    constexpr int JB = KZ <= 3 ? 4 : KZ <= 8 ? 3 : 2, IB = KZ <= 5 ? 4 : KZ <= 8 ? 3 : 2;
    const int jblocks = (fo + JB - 1) / JB, iblocks = (f + IB - 1) / IB;
    const long pchunks = (plane + kThreads - 1) / kThreads;
    const long tiles = pchunks * ((jblocks + kTileJ - 1) / kTileJ) * ((iblocks + kTileI - 1) / kTileI);
    // Planes that fill their last chunk of 256 pencils badly (the 2D benchmark layer: 129 of 256) are walked
    // with a flat (pair block, pencil) index instead of one chunk per workgroup; large planes keep the
    // chunked order, whose super-tiles keep a chunk's spectra in one XCD's L2.
    const int flat = (double)plane < 0.95 * (double)(pchunks * kThreads) ? 1 : 0;
    const long blocks = flat ? ((long)jblocks * iblocks * plane + kThreads - 1) / kThreads : ((tiles + 7) / 8) * 8 * kTileJ * kTileI;
    if (blocks >= 2147483647L) return fail(ZNN_EUNSUPPORTED, "too many edges or pencils for one launch");
    if (vol * 8 >= 4294967296L) return fail(ZNN_EUNSUPPORTED, "a node spectrum of 4 GB or more");
    const dim3 grid((unsigned)blocks);
    if (N % 4 == 0 && tz == 1 && !tuning().fft_wgrad_plain) {
        if (flat)
            ZNN_LAUNCH("pruned DFT of spectral products", s, (k_wgrad_zdft4<KZ, JB, IB, true>), grid, dim3(kThreads), 0,
                       G, I, T, f, fo, N, plane, vol, iblocks);
        else
            ZNN_LAUNCH("pruned DFT of spectral products", s, (k_wgrad_zdft4<KZ, JB, IB, false>), grid, dim3(kThreads), 0,
                       G, I, T, f, fo, N, plane, vol, iblocks);
    } else
        ZNN_LAUNCH("pruned DFT of spectral products", s, (k_wgrad_zdft<KZ, JB, IB>), grid, dim3(kThreads), 0,
                   G, I, T, f, fo, N, tz, plane, vol, iblocks, flat);
    return check_launch("pruned DFT of spectral products");
}

int launch_wgrad_dft(int k, int f, int fo, int N, int tz, long plane, long vol, const float2* G, const float2* I, float2* T,
                     hipStream_t s)
{
    switch (k) {
        case 1: return launch_wgrad_dft_k<1>(f, fo, N, tz, plane, vol, G, I, T, s);
        case 2: return launch_wgrad_dft_k<2>(f, fo, N, tz, plane, vol, G, I, T, s);
        case 3: return launch_wgrad_dft_k<3>(f, fo, N, tz, plane, vol, G, I, T, s);
        case 4: return launch_wgrad_dft_k<4>(f, fo, N, tz, plane, vol, G, I, T, s);
        case 5: return launch_wgrad_dft_k<5>(f, fo, N, tz, plane, vol, G, I, T, s);
        case 6: return launch_wgrad_dft_k<6>(f, fo, N, tz, plane, vol, G, I, T, s);
        case 7: return launch_wgrad_dft_k<7>(f, fo, N, tz, plane, vol, G, I, T, s);
        case 8: return launch_wgrad_dft_k<8>(f, fo, N, tz, plane, vol, G, I, T, s);
        case 9: return launch_wgrad_dft_k<9>(f, fo, N, tz, plane, vol, G, I, T, s);
        case 10: return launch_wgrad_dft_k<10>(f, fo, N, tz, plane, vol, G, I, T, s);
        case 11: return launch_wgrad_dft_k<11>(f, fo, N, tz, plane, vol, G, I, T, s);
        case 12: return launch_wgrad_dft_k<12>(f, fo, N, tz, plane, vol, G, I, T, s);
        case 13: return launch_wgrad_dft_k<13>(f, fo, N, tz, plane, vol, G, I, T, s);
        case 14: return launch_wgrad_dft_k<14>(f, fo, N, tz, plane, vol, G, I, T, s);
        case 15: return launch_wgrad_dft_k<15>(f, fo, N, tz, plane, vol, G, I, T, s);
        default: return launch_wgrad_dft_k<16>(f, fo, N, tz, plane, vol, G, I, T, s);
    }
}

// ---------------------------------------------------------------- launch helpers
int launch_r2c(const float* src, float2* dst, long maps, int sz, int sy, int sx,
               int Nz, int Ny, int Nx, int oz, int oy, int ox, int tz, int ty, int tx, hipStream_t s)
{
    // rows one sample apart along x whose transform length has an instance: one row per thread, in registers
    if (tx == 1 && !tuning().fft_lds_passes && fft_x_reg_supported(Nx) && sx <= Nx - ox) {
        XRegR2C X = {};
        X.src = src; X.dst = dst;
        X.rows = maps * sz * sy;
        X.sz = sz; X.sy = sy; X.sx = sx;
        X.Nz = Nz; X.Ny = Ny; X.Nxh = Nx / 2 + 1;
        X.oz = oz; X.oy = oy; X.ox = ox;
        X.tz = tz; X.ty = ty;
        X.fsy = make_fastdiv((unsigned)sy); X.fsz = make_fastdiv((unsigned)sz);
        return fft_x_r2c_reg(X, Nx, s);
    }
    R2CParams P;
    P.tz = tz; P.ty = ty; P.tx = tx;
    P.src = src; P.dst = dst;
    P.rows = maps * sz * sy;
    P.sz = sz; P.sy = sy; P.sx = sx;
    P.Nz = Nz; P.Ny = Ny; P.Nx = Nx; P.Nxh = Nx / 2 + 1;
    P.oz = oz; P.oy = oy; P.ox = ox;
    int wp = max_row_len(Nx, true);
    if (wp > 33) wp = 33;
    P.W = wp; P.Wp = wp;
    P.rad = factorize(Nx, P.W);
    P.fsx = make_fastdiv((unsigned)sx); P.fnxh = make_fastdiv((unsigned)P.Nxh);
    P.fsy = make_fastdiv((unsigned)sy); P.fsz = make_fastdiv((unsigned)sz);
    const long blocks = (P.rows + 2 * P.W - 1) / (2 * P.W);
    if (blocks >= 2147483647L) return fail(ZNN_EUNSUPPORTED, "too many rows for one launch");
    ZNN_LAUNCH("fft r2c x", s, k_fft_r2c_x, dim3((unsigned)blocks), dim3(kThreads), lds_bytes(Nx, P.Wp), P);
    return check_launch("r2c x pass");
}

int launch_c2r(const float2* src, float* dst, long maps, int Nz, int Ny, int Nx,
               int cz, int cy, int cx, int dz, int dy, int dx, int tx, float scale, hipStream_t s)
{
    if (tx == 1 && !tuning().fft_lds_passes && fft_x_reg_supported(Nx) && dx <= Nx - cx) {
        XRegC2R X = {};
        X.src = src; X.dst = dst;
        X.rows = maps * dz * dy;
        X.cz = cz; X.cy = cy; X.cx = cx;
        X.dz = dz; X.dy = dy; X.dx = dx;
        X.Nz = Nz; X.Ny = Ny; X.Nxh = Nx / 2 + 1;
        X.scale = scale;
        X.fdy = make_fastdiv((unsigned)dy); X.fdz = make_fastdiv((unsigned)dz);
        return fft_x_c2r_reg(X, Nx, s);
    }
    C2RParams P;
    P.tx = tx;
    P.src = src; P.dst = dst;
    P.rows = maps * dz * dy;
    P.cz = cz; P.cy = cy; P.cx = cx;
    P.dz = dz; P.dy = dy; P.dx = dx;
    P.Nz = Nz; P.Ny = Ny; P.Nx = Nx; P.Nxh = Nx / 2 + 1;
    P.scale = scale;
    int wp = max_row_len(Nx, true);
    if (wp > 33) wp = 33;
    P.W = wp; P.Wp = wp;
    P.rad = factorize(Nx, P.W);
    P.fdx = make_fastdiv((unsigned)dx); P.fnxh = make_fastdiv((unsigned)P.Nxh);
    P.fdy = make_fastdiv((unsigned)dy); P.fdz = make_fastdiv((unsigned)dz);
    const long blocks = (P.rows + 2 * P.W - 1) / (2 * P.W);
    if (blocks >= 2147483647L) return fail(ZNN_EUNSUPPORTED, "too many rows for one launch");
    ZNN_LAUNCH("fft c2r x", s, k_fft_c2r_x, dim3((unsigned)blocks), dim3(kThreads), lds_bytes(Nx, P.Wp), P);
    return check_launch("c2r x pass");
}

// Fills the chunking fields and launches.  `P` arrives with everything else set.
int launch_axis(AxisParams P, int dir, hipStream_t s)
{
    if (P.istep < 1) P.istep = 1;
    if (P.ostep < 1) P.ostep = 1;
    if (P.N == 1 && !P.in2 && P.in == P.out && P.in_stride == P.out_stride &&
        P.in_sa == P.out_sa && P.in_sb == P.out_sb && P.in_sc == P.out_sc)
        return ZNN_OK;   // length-1 transform in place: nothing to do
    // extents that fit the register file: one pencil per thread, no LDS
    if (!tuning().fft_lds_passes && !P.in2 && P.istep == 1 && P.ostep == 1 && P.Oc == 1 && P.in_stride == P.L &&
        P.out_stride == P.L && fft_axis_reg_supported(P.N)) {
        RegAxis R = {};
        R.in = P.in; R.out = P.out;
        R.N = P.N; R.i0 = P.i0; R.ni = P.ni; R.o0 = P.o0; R.no = P.no;
        R.stride = P.L; R.L = P.L; R.Oa = P.Oa; R.Ob = P.Ob;
        R.in_sa = P.in_sa; R.in_sb = P.in_sb; R.out_sa = P.out_sa; R.out_sb = P.out_sb;
        if (P.Ob == 1) {    // one run of pencils per outer index: let the threads run across outer indices
            R.Oa = 1; R.Ob = P.Oa;
            R.in_sb = P.in_sa; R.out_sb = P.out_sa;
        }
        if (R.Oa <= 65535 && (long)R.Ob * R.L * R.L < 4294967296L) return fft_axis_reg(R, dir, s);
    }
    // longer pencils that split into two factors of at most 16: two levels, samples in registers at both
    if (!P.in2 && P.istep == 1 && P.ostep == 1 && !tuning().fft_no_two_level && !tuning().fft_lds_passes &&
        fft_axis_two_level_supported(P.N)) {
        TwoLevelAxis T = {};
        T.in = P.in; T.out = P.out;
        T.N = P.N; T.i0 = P.i0; T.ni = P.ni; T.o0 = P.o0; T.no = P.no;
        T.in_stride = P.in_stride; T.out_stride = P.out_stride;
        T.L = P.L; T.Oa = P.Oa; T.Ob = P.Ob; T.Oc = P.Oc;
        T.in_sa = P.in_sa; T.in_sb = P.in_sb; T.in_sc = P.in_sc;
        T.out_sa = P.out_sa; T.out_sb = P.out_sb; T.out_sc = P.out_sc;
        if ((long)P.Oa * P.Ob * P.Oc * ((P.L + 15) / 16) < 4294967296L / std::max(std::max(P.Ob, P.Oc), (P.L + 15) / 16))
            return fft_axis_two_level(T, dir, s);
    }
    // chunk width: a whole line when it fits, else a multiple of 16 pencils (128 bytes) so
    // that every chunk starts on a cache-line boundary
    int wmax = max_row_len(P.N, false) > 63 ? 63 : max_row_len(P.N, false);
    if (P.L > wmax && wmax >= 16) wmax = wmax >= 48 ? 32 : (wmax / 16) * 16;
    const int chunks = (P.L + wmax - 1) / wmax;
    P.chunks = chunks;
    P.W = P.L > wmax ? wmax : P.L;
    P.Wp = P.W | 1;
    P.rad = factorize(P.N, P.W);
    P.fchunks = make_fastdiv((unsigned)chunks);
    P.foc = make_fastdiv((unsigned)P.Oc);
    P.fob = make_fastdiv((unsigned)P.Ob);
    const long blocks = (long)P.Oa * P.Ob * P.Oc * chunks;
    // the block index is taken apart with multiply-high divisions, exact while index * divisor < 2^32
    const long dmax = std::max((long)chunks, std::max((long)P.Oc, (long)P.Ob));
    if (blocks * dmax >= 4294967296L) return fail(ZNN_EUNSUPPORTED, "too many pencils for one launch");
    const size_t lds = lds_bytes(P.N, P.Wp);
    const dim3 grid((unsigned)blocks), block(kThreads);
    if (P.in2) {
        if (dir > 0) ZNN_LAUNCH("fft axis inverse of product", s, (k_fft_axis<+1, true>), grid, block, lds, P);
        else         ZNN_LAUNCH("fft axis forward of product", s, (k_fft_axis<-1, true>), grid, block, lds, P);
    } else {
        if (dir > 0) ZNN_LAUNCH("fft axis inverse", s, (k_fft_axis<+1, false>), grid, block, lds, P);
        else         ZNN_LAUNCH("fft axis forward", s, (k_fft_axis<-1, false>), grid, block, lds, P);
    }
    return check_launch("strided FFT pass");
}

// Forward 3D transform of `maps` real volumes of extents (sz,sy,sx) embedded at
// offset (oz,oy,ox) of the (Nz,Ny,Nx) volume.  Neighbouring source samples land
// (tz,ty,tx) voxels apart: 1 for images, the sparsity for kernels, whose taps are
// spread out with zeros between them (Section 2, sparse convolution).
int forward3d(const Geom& g, const float* src, float2* spec, long maps, int sz, int sy, int sx,
              int oz, int oy, int ox, int tz, int ty, int tx, hipStream_t s)
{
    const long plane = (long)g.Ny * g.Nxh, vol = g.svol();
    if (maps > 2147483647L) return fail(ZNN_EUNSUPPORTED, "too many maps");
    // equal x and y transform lengths with register transforms: both passes in one launch
    const bool fused = g.Ny == g.Nx && g.Ny > 1 && tx == 1 && ty == 1 && !tuning().fft_lds_passes && !tuning().fft_no_fused_xy &&
                       fft_xy_reg_supported(g.Nx) && oy + sy <= g.Ny && ox + sx <= g.Nx;
    int rc;
    if (fused) {
        XYFwd F = {};
        F.src = src; F.dst = spec;
        F.planes = maps * sz;
        F.sz = sz; F.sy = sy; F.sx = sx;
        F.Nz = g.Nz; F.oz = oz; F.oy = oy; F.ox = ox; F.tz = tz;
        rc = fft_xy_fwd_reg(F, g.Nx, s);
    } else {
        rc = launch_r2c(src, spec, maps, sz, sy, sx, g.Nz, g.Ny, g.Nx, oz, oy, ox, tz, ty, tx, s);
    }
    if (rc != ZNN_OK) return rc;
    AxisParams P = {};
    // y: only the sz planes that hold data; rows oy + e*ty, e < sy, are non-zero
    P.in = spec + oz * plane; P.in2 = nullptr; P.out = spec + oz * plane;
    P.N = g.Ny; P.i0 = oy; P.ni = sy; P.o0 = 0; P.no = g.Ny;
    P.istep = ty; P.ostep = 1;
    P.in_stride = P.out_stride = g.Nxh;
    P.L = g.Nxh;
    P.Oa = (int)maps; P.Ob = sz; P.Oc = 1;
    P.in_sa = P.out_sa = vol; P.in_sb = P.out_sb = plane * tz; P.in_sc = P.out_sc = 0;
    if (g.Ny != 1 && !fused) {
        // 2D volumes with few non-zero rows (kernels): the y transform is a pruned DFT
        if (g.Nz == 1 && sy <= kMaxPruned && sy < g.Ny) rc = launch_expand(sy, spec, maps, g.Ny, oy, ty, g.Nxh, vol, s);
        else rc = launch_axis(P, -1, s);
        if (rc != ZNN_OK) return rc;
    }
    // z: planes oz + e*tz, e < sz, are non-zero
    P.in = spec; P.out = spec;
    P.N = g.Nz; P.i0 = oz; P.ni = sz; P.o0 = 0; P.no = g.Nz;
    P.istep = tz;
    P.in_stride = P.out_stride = plane;
    P.L = (int)plane;
    P.Oa = (int)maps; P.Ob = 1; P.Oc = 1;
    P.in_sb = P.out_sb = 0;
    if (g.Nz == 1) return ZNN_OK;
    if (sz <= kMaxPruned && sz < g.Nz) return launch_expand(sz, spec, maps, g.Nz, oz, tz, plane, vol, s);
    return launch_axis(P, -1, s);
}

// Inverse 3D transform of `maps` spectra (destroyed) to real volumes cropped to
// [c, c+d) per axis and scaled by 1/(Nz Ny Nx).  z_done: the rows [cz, cz + dz) along z hold
// the inverse transform along z already (the multiply-accumulate applied it).
int inverse3d(const Geom& g, float2* spec, float* dst, long maps, int cz, int cy, int cx,
              int dz, int dy, int dx, bool z_done, hipStream_t s)
{
    const long plane = (long)g.Ny * g.Nxh, vol = g.svol();
    if (maps > 2147483647L) return fail(ZNN_EUNSUPPORTED, "too many maps");
    int rc;
    AxisParams P = {};
    P.in = spec; P.in2 = nullptr; P.out = spec;
    P.N = g.Nz; P.i0 = 0; P.ni = g.Nz; P.o0 = cz; P.no = dz;
    P.in_stride = P.out_stride = plane;
    P.L = (int)plane;
    P.Oa = (int)maps; P.Ob = 1; P.Oc = 1;
    P.in_sa = P.out_sa = vol;
    if (g.Nz != 1 && !z_done) { rc = launch_axis(P, +1, s); if (rc != ZNN_OK) return rc; }
    const float scale = (float)(1.0 / ((double)g.Nz * g.Ny * g.Nx));
    if (g.Ny == g.Nx && g.Ny > 1 && !tuning().fft_lds_passes && !tuning().fft_no_fused_xy && fft_xy_reg_supported(g.Nx) &&
        cy + dy <= g.Ny && cx + dx <= g.Nx) {
        XYInv B = {};
        B.src = spec; B.dst = dst;
        B.planes = maps * dz;
        B.dz = dz; B.dy = dy; B.dx = dx;
        B.Nz = g.Nz; B.cz = cz; B.cy = cy; B.cx = cx;
        B.scale = scale;
        return fft_xy_inv_reg(B, g.Nx, s);
    }
    P.in = spec + cz * plane; P.out = spec + cz * plane;
    P.N = g.Ny; P.i0 = 0; P.ni = g.Ny; P.o0 = cy; P.no = dy;
    P.in_stride = P.out_stride = g.Nxh;
    P.L = g.Nxh;
    P.Oa = (int)maps; P.Ob = dz; P.Oc = 1;
    P.in_sb = P.out_sb = plane;
    if (g.Ny != 1) { rc = launch_axis(P, +1, s); if (rc != ZNN_OK) return rc; }
    return launch_c2r(spec, dst, maps, g.Nz, g.Ny, g.Nx, cz, cy, cx, dz, dy, dx, 1, scale, s);
}

// Layers whose kernel spectra can be kept as half spectra (transformed along the fast axes
// only) and expanded inside the multiply-accumulate: the slowest non-trivial axis must have a
// length divisible by 4, few taps, and taps one voxel apart.  `min_blocks`: fewest workgroups
// per group of result nodes for which the folded kernel is worth launching.
Fold fold_search(const Geom& g, long min_blocks)
{
    Fold F = {false, 0, 0, 0, 0};
    if (g.Nz > 1) { F.N = g.Nz; F.taps = g.kz; F.P = g.Ny * g.Nxh; F.on = g.spz == 1; }
    else if (g.Ny > 1) { F.N = g.Ny; F.taps = g.ky; F.P = g.Nxh; F.on = g.spy == 1; }
    F.on = F.on && F.N % 4 == 0 && F.taps <= kMaxFoldedTaps && F.taps < F.N;
    if (!F.on) return F;
    // the folded kernel has about (N/4/z0) * P threads per group of result nodes: small layers
    // would leave most of the chip idle, they keep the full spectra
    const int nmin = g.f < g.fo ? g.f : g.fo;
    // Four base frequencies per thread reuse every loaded value most but leave the fewest
    // threads: they win on layers with thousands of workgroups (config 5: 30.0 ms against
    // 31.2 ms), two win below that (config 2: 1.26 against 1.33 ms; config 4: 1.54 against
    // 1.76 ms), one is the fallback for extents not divisible by 8.
    const int pin = tuning().fft_mac_z0;
    auto blocks_of = [&](int z0) {
        const int G = fft_mac_group(z0);
        return (long)((F.P + 63) / 64) * ((F.N / 4 / z0 + 3) / 4) * ((nmin + G - 1) / G);
    };
    const bool big = (F.N / 4) % 4 == 0 && blocks_of(4) >= 2048;
    const int order[3] = {big ? 4 : 2, big ? 2 : 4, 1};
    F.z0 = 0;
    for (int k = 0; k < 3 && !F.z0; ++k) {
        const int z0 = order[k];
        if ((pin && z0 != pin) || (F.N / 4) % z0) continue;
        if (blocks_of(z0) >= min_blocks) F.z0 = z0;
    }
    F.on = F.z0 != 0;
    return F;
}

// cz, dz: the rows along z that the inverse transform of the result has to deliver; *z_done: they hold the
// inverse transform along z already (3D layers whose folded multiply-accumulate owns the whole axis per wave).
int launch_mac(bool backward, const Geom& g, const Fold& F, const float2* What, const float2* a, float2* b,
               int cz, int dz, bool* z_done, hipStream_t s)
{
    *z_done = false;
    if (F.on) {
        if (!tuning().fft_mac_valu && fft_mac_mfma_supported(F.taps, F.N, F.P)) {
            const bool inv = g.Nz > 1 && !tuning().fft_no_mac_inverse &&
                             fft_mac_mfma_can_invert(F.taps, F.N, F.P, backward ? g.f : g.fo);
            *z_done = inv;
            return fft_mac_mfma(backward, F.taps, g.f, g.fo, F.N, F.P, What, a, b, cz, inv ? dz : 0, s);
        }
        return fft_mac_fused(backward, F.taps, F.z0, g.f, g.fo, F.N, F.P, What, a, b, s);
    }
    const long svol = g.svol();
    const int outs = backward ? g.f : g.fo;
    const int V = (svol % 2 == 0) ? 2 : 1;
    const long threads = (svol + V - 1) / V;
    dim3 grid((unsigned)((threads + kThreads - 1) / kThreads), (unsigned)((outs + kMacGroup - 1) / kMacGroup));
    if (backward) {
        if (V == 2) ZNN_LAUNCH("spectral mac backward", s, (k_mac<true, 2>), grid, dim3(kThreads), 0, g.f, g.fo, svol, What, a, b);
        else        ZNN_LAUNCH("spectral mac backward", s, (k_mac<true, 1>), grid, dim3(kThreads), 0, g.f, g.fo, svol, What, a, b);
    } else {
        if (V == 2) ZNN_LAUNCH("spectral mac forward", s, (k_mac<false, 2>), grid, dim3(kThreads), 0, g.f, g.fo, svol, What, a, b);
        else        ZNN_LAUNCH("spectral mac forward", s, (k_mac<false, 1>), grid, dim3(kThreads), 0, g.f, g.fo, svol, What, a, b);
    }
    return check_launch("spectral multiply-accumulate");
}

}  // namespace

// ---------------------------------------------------------------- public (library-internal) entry points
Fold fold_full() { return Fold{false, 0, 0, 0, 0}; }
Fold fold_default(const Geom& g) { return fold_search(g, 128); }
Fold fold_forced(const Geom& g) { return fold_search(g, 1); }

size_t fft_spectra_bytes(const Geom& g, const Fold& F)
{
    if (F.on) return align256(sizeof(float2) * (size_t)g.f * g.fo * F.taps * F.P);
    return align256(sizeof(float2) * (size_t)g.f * g.fo * g.svol());
}

FftWorkspace fft_workspace(const Geom& g, const Fold& F, int pass, bool resident)
{
    FftWorkspace w = {};
    size_t o = 0;
    const size_t spec = sizeof(float2) * (size_t)g.svol();
    if (pass == ZNN_PASS_FWD || pass == ZNN_PASS_BWD) {
        const int na = pass == ZNN_PASS_FWD ? g.f : g.fo;
        const int nb = pass == ZNN_PASS_FWD ? g.fo : g.f;
        w.off_a = o; o += align256(spec * na);
        w.off_b = o; o += align256(spec * nb);
        w.off_w = o;
        if (!resident) o += fft_spectra_bytes(g, F);
    } else {
        const size_t pairs = (size_t)g.f * g.fo;
        w.off_a = o; o += align256(spec * g.f);
        w.off_b = o; o += align256(spec * g.fo);
        w.off_t1 = o; o += align256(sizeof(float2) * pairs * g.kz * g.Ny * g.Nxh);
        w.off_t2 = o; o += align256(sizeof(float2) * pairs * g.kz * g.ky * g.Nxh);
    }
    w.total = o;
    return w;
}

int fft_kernel_spectra(const Geom& g, const Fold& F, const float* w, float2* What, hipStream_t s)
{
    if (F.on) {
        // half spectra [pair][tap][P]: x (and, in 3D, y) transforms of the planes that hold taps
        const long pairs = (long)g.f * g.fo;
        if (pairs * F.taps > 2147483647L) return fail(ZNN_EUNSUPPORTED, "too many kernel planes");
        if (g.Nz == 1)
            return launch_r2c(w, What, pairs, 1, g.ky, g.kx, 1, g.ky, g.Nx, 0, 0, 0, 1, 1, g.spx, s);
        if (g.Ny == g.Nx && g.Ny > 1 && g.spy == 1 && g.spx == 1 && !tuning().fft_lds_passes && !tuning().fft_no_fused_xy &&
            fft_xy_reg_supported(g.Nx)) {
            XYFwd F = {};
            F.src = w; F.dst = What;
            F.planes = pairs * g.kz;
            F.sz = g.kz; F.sy = g.ky; F.sx = g.kx;
            F.Nz = g.kz; F.oz = 0; F.oy = 0; F.ox = 0; F.tz = 1;
            return fft_xy_fwd_reg(F, g.Nx, s);
        }
        int rc = launch_r2c(w, What, pairs, g.kz, g.ky, g.kx, g.kz, g.Ny, g.Nx, 0, 0, 0, 1, g.spy, g.spx, s);
        if (rc != ZNN_OK || g.Ny == 1) return rc;
        const long plane = (long)g.Ny * g.Nxh;
        AxisParams P = {};
        P.in = What; P.in2 = nullptr; P.out = What;
        P.N = g.Ny; P.i0 = 0; P.ni = g.ky; P.o0 = 0; P.no = g.Ny;
        P.istep = g.spy; P.ostep = 1;
        P.in_stride = P.out_stride = g.Nxh;
        P.L = g.Nxh;
        P.Oa = (int)(pairs * g.kz); P.Ob = 1; P.Oc = 1;
        P.in_sa = P.out_sa = plane;
        return launch_axis(P, -1, s);
    }
    return forward3d(g, w, What, (long)g.f * g.fo, g.kz, g.ky, g.kx, 0, 0, 0, g.spz, g.spy, g.spx, s);
}

int fft_fwd(const Geom& g, const Fold& F, const float* in, const float* w, const float2* resident, float* out,
            void* ws, float2* memo_in, hipStream_t s)
{
    const FftWorkspace L = fft_workspace(g, F, ZNN_PASS_FWD, resident != nullptr);
    float2* Ihat = memo_in ? memo_in : (float2*)((char*)ws + L.off_a);
    float2* Ohat = (float2*)((char*)ws + L.off_b);
    const float2* What = resident;
    int rc = forward3d(g, in, Ihat, g.f, g.nz, g.ny, g.nx, 0, 0, 0, 1, 1, 1, s);
    if (rc != ZNN_OK) return rc;
    if (!What) {
        float2* wbuf = (float2*)((char*)ws + L.off_w);
        rc = fft_kernel_spectra(g, F, w, wbuf, s);
        if (rc != ZNN_OK) return rc;
        What = wbuf;
    }
    bool z_done;
    rc = launch_mac(false, g, F, What, Ihat, Ohat, g.spz * (g.kz - 1), g.oz, &z_done, s);
    if (rc != ZNN_OK) return rc;
    return inverse3d(g, Ohat, out, g.fo, g.spz * (g.kz - 1), g.spy * (g.ky - 1), g.spx * (g.kx - 1),
                     g.oz, g.oy, g.ox, z_done, s);
}

int fft_bwd(const Geom& g, const Fold& F, const float* gout, const float* w, const float2* resident, float* gin,
            void* ws, float2* memo_gout, hipStream_t s)
{
    const FftWorkspace L = fft_workspace(g, F, ZNN_PASS_BWD, resident != nullptr);
    float2* Ghat = memo_gout ? memo_gout : (float2*)((char*)ws + L.off_a);
    float2* Ginhat = (float2*)((char*)ws + L.off_b);
    const float2* What = resident;
    int rc = forward3d(g, gout, Ghat, g.fo, g.oz, g.oy, g.ox, g.spz * (g.kz - 1), g.spy * (g.ky - 1), g.spx * (g.kx - 1),
                       1, 1, 1, s);
    if (rc != ZNN_OK) return rc;
    if (!What) {
        float2* wbuf = (float2*)((char*)ws + L.off_w);
        rc = fft_kernel_spectra(g, F, w, wbuf, s);
        if (rc != ZNN_OK) return rc;
        What = wbuf;
    }
    bool z_done;
    rc = launch_mac(true, g, F, What, Ghat, Ginhat, 0, g.nz, &z_done, s);
    if (rc != ZNN_OK) return rc;
    return inverse3d(g, Ginhat, gin, g.f, 0, 0, 0, g.nz, g.ny, g.nx, z_done, s);
}

int fft_wgrad(const Geom& g, const float* in, const float* gout, float* gw, void* ws, hipStream_t s)
{
    const FftWorkspace L = fft_workspace(g, fold_full(), ZNN_PASS_WGRAD, false);
    float2* Ihat = (float2*)((char*)ws + L.off_a);
    float2* Ghat = (float2*)((char*)ws + L.off_b);
    int rc = forward3d(g, in, Ihat, g.f, g.nz, g.ny, g.nx, 0, 0, 0, 1, 1, 1, s);
    if (rc != ZNN_OK) return rc;
    rc = forward3d(g, gout, Ghat, g.fo, g.oz, g.oy, g.ox, g.spz * (g.kz - 1), g.spy * (g.ky - 1), g.spx * (g.kx - 1),
                       1, 1, 1, s);
    if (rc != ZNN_OK) return rc;
    return fft_wgrad_from_spectra(g, Ihat, Ghat, gw, ws, s);
}

// Kernel gradient from node spectra that already exist (memoized by the forward and
// backward pass, or just computed): gw = crop[0,k) IFFT( G_s^[j] conj(I^[i]) ).
int fft_wgrad_from_spectra(const Geom& g, const float2* Ihat, const float2* Ghat, float* gw, void* ws,
                           hipStream_t s)
{
    const FftWorkspace L = fft_workspace(g, fold_full(), ZNN_PASS_WGRAD, false);
    float2* T1 = (float2*)((char*)ws + L.off_t1);
    float2* T2 = (float2*)((char*)ws + L.off_t2);
    int rc = ZNN_OK;
    const long plane = (long)g.Ny * g.Nxh, vol = g.svol();
    if (g.Nz == 1 && g.Ny > 1 && g.ky <= kMaxPruned) {
        // 2D: the y axis is the first one contracted; its ky outputs land directly in T2
        rc = launch_wgrad_dft(g.ky, g.f, g.fo, g.Ny, g.spy, g.Nxh, vol, Ghat, Ihat, T2, s);
        if (rc != ZNN_OK) return rc;
    } else {
        // z: product G^[j] conj(I^[i]); only z in [0, kz) is kept
        AxisParams P = {};
        P.in = Ghat; P.in2 = Ihat; P.out = T1;
        P.N = g.Nz; P.i0 = 0; P.ni = g.Nz; P.o0 = 0; P.no = g.kz;
        P.ostep = g.spz;                    // tap a is lag a*s of the correlation
        P.in_stride = plane; P.out_stride = plane;
        P.L = (int)plane;
        P.Oa = g.fo; P.Ob = g.f; P.Oc = 1;
        P.in_sa = vol; P.in_sb = 0;
        P.in2_sa = 0; P.in2_sb = vol;
        P.out_sa = (long)g.f * g.kz * plane; P.out_sb = (long)g.kz * plane;
        if (g.kz <= kMaxPruned) rc = launch_wgrad_dft(g.kz, g.f, g.fo, g.Nz, g.spz, plane, vol, Ghat, Ihat, T1, s);
        else rc = launch_axis(P, +1, s);
        if (rc != ZNN_OK) return rc;
        // y: only y in [0, ky) is kept, written compactly
        P = AxisParams{};
        P.in = T1; P.in2 = nullptr; P.out = T2;
        P.N = g.Ny; P.i0 = 0; P.ni = g.Ny; P.o0 = 0; P.no = g.ky;
        P.ostep = g.spy;
        P.in_stride = g.Nxh; P.out_stride = g.Nxh;
        P.L = g.Nxh;
        P.Oa = g.fo * g.f; P.Ob = g.kz; P.Oc = 1;
        P.in_sa = (long)g.kz * plane; P.in_sb = plane;
        P.out_sa = (long)g.kz * g.ky * g.Nxh; P.out_sb = (long)g.ky * g.Nxh;
        if (g.ky <= kMaxPruned && !tuning().fft_wgrad_plain)
            rc = launch_prune(g.ky, T1, T2, (long)g.fo * g.f * g.kz, g.Ny, g.Nxh, g.spy, s);
        else
            rc = launch_axis(P, +1, s);
        if (rc != ZNN_OK) return rc;
    }
    const float scale = (float)(1.0 / ((double)g.Nz * g.Ny * g.Nx));
    return launch_c2r(T2, gw, (long)g.f * g.fo, g.kz, g.ky, g.Nx, 0, 0, 0, g.kz, g.ky, g.kx, g.spx, scale, s);
}

}  // namespace znn
