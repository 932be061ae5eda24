// x-axis passes of the 3D transforms (real -> complex and back) with one row per thread, the row's
// transform in registers (templates; included by the fft_x_reg_*.hip translation units).
//
// Along x the elements of a pencil are contiguous in memory, so a thread cannot simply load its own
// row (64 lanes would touch 64 different rows).  A wave therefore moves its 64 rows between global
// memory and a private LDS region row by row -- one wave-wide, fully coalesced access per row and
// 64-float segment, global -> LDS without passing registers on the way in -- and each lane then
// reads, resp. writes, its own row there (odd row pitch: no bank conflicts).  Waves never wait for
// each other: there is no workgroup barrier in these kernels.
//
// A real row of N = 2 H samples is transformed as ONE complex transform of length H on
// z[m] = a[2m] + i a[2m+1] (fully unrolled Stockham passes of fft_reg_impl.h, compile-time twiddles):
//     forward   X[k] = 1/2 [ (Z[k] + conj Z[H-k]) - i w^k (Z[k] - conj Z[H-k]) ],  w = exp(-2 pi i / N), k = 0..H
//     inverse   Z[k] = (X[k] + conj X[H-k]) + i w^-k (X[k] - conj X[H-k]),  z = IFFT_H(Z)  (N times the samples)
// Rows shorter than N are zero-extended (sx samples from offset ox), cropped on the way back.
// Instantiated for N = 2 H with H a 5-smooth extent from 8 to 96; other extents, sparse kernels
// (samples more than one voxel apart along x) and N > 192 take the LDS passes in fft.hip.
#pragma once

#include "fft_reg_impl.h"

namespace znn {

namespace {

constexpr int kXWaves = 4;
constexpr int kStageFloats = 64 * 66;           // 64 rows x (pitch 65 floats | pitch 33 complex)

typedef __attribute__((address_space(1))) const void* global_cptr;
typedef __attribute__((address_space(3))) void* lds_ptr;

__device__ __forceinline__ void lds_wait() { __builtin_amdgcn_s_waitcnt(0xC07F); }      // lgkmcnt(0)

// Spectrum row (in complex elements) of source / result row `row0 + t`, t = lane: rows are counted
// (map, z, y) with extents (., ez, ey); z and y are placed at z * tz + oz, y * ty + oy of the volume.
__device__ __forceinline__ long spectrum_row(long row0, int t, int ez, int ey, FastDiv fey, FastDiv fez,
                                             int Nz, int Ny, int Nxh, int oz, int oy, int tz, int ty)
{
    const long map0 = row0 / ((long)ey * ez);                       // once per wave (uniform)
    const int rem0 = (int)(row0 - map0 * ((long)ey * ez));
    const int z0 = rem0 / ey, y0 = rem0 - z0 * ey;
    const int yy = y0 + t;
    const int zc = (int)fdiv((unsigned)yy, fey);
    const int y = yy - zc * ey;
    const int zz = z0 + zc;
    const int mc = (int)fdiv((unsigned)zz, fez);
    const int z = zz - mc * ez;
    return (((map0 + mc) * Nz + z * tz + oz) * Ny + (y * ty + oy)) * (long)Nxh;
}

template <int H>
__global__ void __launch_bounds__(64 * kXWaves) k_fft_r2c_x_reg(XRegR2C P)
{
    constexpr int N = 2 * H, NXH = H + 1;
    __shared__ __attribute__((aligned(16))) float stage[kXWaves][kStageFloats];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    float* st = stage[wave];
    if (P.rows < 0) st[lane] = P.src[lane];         // never taken: tells the optimizer that LDS holds data
    const long row0 = ((long)blockIdx.x * kXWaves + wave) * 64;
    if (row0 >= P.rows) return;                     // wave-uniform
    const int nrows = (int)min((long)64, P.rows - row0);
    const bool padded = P.ox != 0 || P.sx != N;     // lanes outside the samples never load: their words must hold zeros

    float2 x[H], y[H];
#pragma unroll
    for (int c = 0; c * 64 < N; ++c) {
        if (c == 0 || padded) {
            for (int i = lane; i < 64 * 65; i += 64) st[i] = 0.f;
        }
        lds_wait();
        const int s = c * 64 + lane - P.ox;
        const bool lvalid = c * 64 + lane < N && s >= 0 && s < P.sx;
        const float* rp = P.src + row0 * P.sx + s;
        for (int r = 0; r < nrows; ++r) {
            if (lvalid) __builtin_amdgcn_global_load_lds((global_cptr)(rp + (long)r * P.sx), (lds_ptr)(st + r * 65), 4, 0, 0);
        }
        __builtin_amdgcn_s_waitcnt(0);              // the rows have landed
#pragma unroll
        for (int xx = 0; xx < 64; xx += 2) {
            if (c * 64 + xx < N) x[(c * 64 + xx) / 2] = make_float2(st[lane * 65 + xx], st[lane * 65 + xx + 1]);
        }
    }

    passes<H, -1, H, 1>(x, y);
    constexpr bool in_y = (count_passes(H) % 2) == 1;
    float2 (&Z)[H] = in_y ? y : x;
    float2 (&X)[H] = in_y ? x : y;                  // the other array takes X[0..H-1]; X[H] apart
    float2 XH;
    {
        // k = 0 and k = H: Z[H] = Z[0], w^0 = 1, w^H = -i ... both reduce to sums of Re and Im of Z[0]
        const float2 z0 = Z[0];
        X[0] = make_float2(z0.x + z0.y, 0.f);
        XH = make_float2(z0.x - z0.y, 0.f);
    }
#pragma unroll
    for (int k = 1; k < H; ++k) {
        const float2 a = Z[k], b = Z[H - k];
        const float2 e = make_float2(a.x + b.x, a.y - b.y);            // Z[k] + conj Z[H-k]
        const float2 d = make_float2(a.x - b.x, a.y + b.y);            // Z[k] - conj Z[H-k]
        constexpr float dummy = 0.f; (void)dummy;
        const float wc = TwTable<N>::t.c[k], ws = -TwTable<N>::t.s[k]; // w^k = exp(-2 pi i k / N)
        // -i w^k d = -i (wc + i ws)(d.x + i d.y) = (wc d.y + ws d.x) + i (ws d.y - wc d.x)
        X[k] = make_float2(0.5f * (e.x + wc * d.y + ws * d.x), 0.5f * (e.y + ws * d.y - wc * d.x));
    }

    const long myrow = spectrum_row(row0, lane, P.sz, P.sy, P.fsy, P.fsz, P.Nz, P.Ny, P.Nxh, P.oz, P.oy, P.tz, P.ty);
    const int rlo = (int)(myrow & 0xffffffffL), rhi = (int)(myrow >> 32);
    float2* st2 = reinterpret_cast<float2*>(st);    // rows of 32 complex, pitch 33
    const int half = lane >> 5, kk = lane & 31;
#pragma unroll
    for (int c = 0; c * 32 < NXH; ++c) {
        lds_wait();
#pragma unroll
        for (int q = 0; q < 32; ++q) {
            const int k = c * 32 + q;
            if (k < H) st2[lane * 33 + q] = X[k];
            else if (k == H) st2[lane * 33 + q] = XH;
        }
        const bool kvalid = c * 32 + kk < NXH;
        for (int r = 0; r < nrows; r += 2) {
            const long b0 = ((long)__builtin_amdgcn_readlane(rhi, r) << 32) | (unsigned)__builtin_amdgcn_readlane(rlo, r);
            const int r1 = min(r + 1, 63);
            const long b1 = ((long)__builtin_amdgcn_readlane(rhi, r1) << 32) | (unsigned)__builtin_amdgcn_readlane(rlo, r1);
            const float2 v = st2[(r + half) * 33 + kk];
            if (kvalid && r + half < nrows) P.dst[(half ? b1 : b0) + c * 32 + kk] = v;
        }
    }
}

template <int H>
__global__ void __launch_bounds__(64 * kXWaves) k_fft_c2r_x_reg(XRegC2R P)
{
    constexpr int N = 2 * H, NXH = H + 1;
    __shared__ __attribute__((aligned(16))) float stage[kXWaves][kStageFloats];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    float* st = stage[wave];
    if (P.rows < 0) st[lane] = P.dst[lane];         // never taken: tells the optimizer that LDS holds data
    const long row0 = ((long)blockIdx.x * kXWaves + wave) * 64;
    if (row0 >= P.rows) return;
    const int nrows = (int)min((long)64, P.rows - row0);

    const long myrow = spectrum_row(row0, lane, P.dz, P.dy, P.fdy, P.fdz, P.Nz, P.Ny, P.Nxh, P.cz, P.cy, 1, 1);
    const int rlo = (int)(myrow & 0xffffffffL), rhi = (int)(myrow >> 32);
    const float* sf = reinterpret_cast<const float*>(P.src);

    float2 X[NXH];
#pragma unroll
    for (int c = 0; c * 32 < NXH; ++c) {
        lds_wait();
        const bool lvalid = c * 64 + lane < 2 * NXH;
        for (int r = 0; r < nrows; ++r) {
            const long b = ((long)__builtin_amdgcn_readlane(rhi, r) << 32) | (unsigned)__builtin_amdgcn_readlane(rlo, r);
            if (lvalid) __builtin_amdgcn_global_load_lds((global_cptr)(sf + (b + c * 32) * 2 + lane), (lds_ptr)(st + r * 65), 4, 0, 0);
        }
        __builtin_amdgcn_s_waitcnt(0);
#pragma unroll
        for (int q = 0; q < 32; ++q)
            if (c * 32 + q < NXH) X[c * 32 + q] = make_float2(st[lane * 65 + 2 * q], st[lane * 65 + 2 * q + 1]);
    }

    float2 x[H], y[H];
    // the imaginary parts of the DC and Nyquist bins of a real line are taken as zero
    x[0] = make_float2(X[0].x + X[H].x, X[0].x - X[H].x);
#pragma unroll
    for (int k = 1; k < H; ++k) {
        const float2 a = X[k], b = X[H - k];
        const float2 e = make_float2(a.x + b.x, a.y - b.y);            // X[k] + conj X[H-k]
        const float2 d = make_float2(a.x - b.x, a.y + b.y);            // X[k] - conj X[H-k]
        const float wc = TwTable<N>::t.c[k], ws = TwTable<N>::t.s[k];  // w^-k = exp(+2 pi i k / N)
        // i w^-k d = i (wc + i ws)(d.x + i d.y) = -(wc d.y + ws d.x) + i (wc d.x - ws d.y)
        x[k] = make_float2(e.x - wc * d.y - ws * d.x, e.y + wc * d.x - ws * d.y);
    }
    passes<H, +1, H, 1>(x, y);
    constexpr bool in_y = (count_passes(H) % 2) == 1;
    float2 (&z)[H] = in_y ? y : x;

    float* drow = P.dst + row0 * P.dx;
#pragma unroll
    for (int c = 0; c * 64 < N; ++c) {
        lds_wait();
#pragma unroll
        for (int xx = 0; xx < 64; xx += 2) {
            if (c * 64 + xx < N) {
                st[lane * 65 + xx] = P.scale * z[(c * 64 + xx) / 2].x;
                st[lane * 65 + xx + 1] = P.scale * z[(c * 64 + xx) / 2].y;
            }
        }
        const int s = c * 64 + lane - P.cx;
        const bool lvalid = c * 64 + lane < N && s >= 0 && s < P.dx;
        for (int r = 0; r < nrows; ++r) {
            const float v = st[r * 65 + lane];
            if (lvalid) drow[(long)r * P.dx + s] = v;
        }
    }
}

template <int H>
int launch_x_r2c(const XRegR2C& P, hipStream_t s)
{
    const long blocks = (P.rows + 64 * kXWaves - 1) / (64 * kXWaves);
    if (blocks >= 2147483647L) return fail(ZNN_EUNSUPPORTED, "too many rows for one launch");
    ZNN_LAUNCH("fft r2c x (registers)", s, (k_fft_r2c_x_reg<H>), dim3((unsigned)blocks), dim3(64 * kXWaves), 0, P);
    return check_launch("r2c x pass");
}

template <int H>
int launch_x_c2r(const XRegC2R& P, hipStream_t s)
{
    const long blocks = (P.rows + 64 * kXWaves - 1) / (64 * kXWaves);
    if (blocks >= 2147483647L) return fail(ZNN_EUNSUPPORTED, "too many rows for one launch");
    ZNN_LAUNCH("fft c2r x (registers)", s, (k_fft_c2r_x_reg<H>), dim3((unsigned)blocks), dim3(64 * kXWaves), 0, P);
    return check_launch("c2r x pass");
}

template <int H>
int launch_x(const XRegR2C* F, const XRegC2R* B, hipStream_t s)
{
    return F ? launch_x_r2c<H>(*F, s) : launch_x_c2r<H>(*B, s);
}

}  // namespace

}  // namespace znn
