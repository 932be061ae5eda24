// x and y passes of a 3D transform in ONE launch, for volumes whose x and y transform lengths are
// equal (templates; included by the fft_xy_reg_*.hip translation units).
//
// A workgroup of two waves owns one (map, z) plane, which fits LDS (N = 96: 37 KiB):
//   forward  the plane's real rows travel global -> LDS (coalesced, no registers); one thread per row
//            transforms its row in registers (half-length complex transform of the real row, as in
//            fft_x_reg_impl.h) and writes the N/2+1 coefficients back to LDS as [y][k]; one thread per
//            column k then runs the length-N transform along y in registers and stores the column,
//            lanes side by side along k (contiguous in the spectrum).
//   inverse  the mirror image: columns in (coalesced along k), y transform in registers, rows through
//            LDS, half-length inverse per row, real rows out.
// The spectrum makes one trip through HBM instead of two, and two launches become one.  Rows and
// columns known to be zero (padding; the few rows of a kernel) are neither read nor transformed, rows
// outside the crop are not produced.
#pragma once

#include "fft_x_reg_impl.h"

namespace znn {

namespace {

constexpr int kXYThreads = 128;

template <int N> struct XYLayout {
    static constexpr int H = N / 2, NXH = H + 1;
    static constexpr int KP = NXH | 1;              // complex row pitch (odd)
    // real row pitch.  N divisible by 4: N + 2, so that rows stay 8-byte aligned (a thread reads its row as
    // pairs) while RP / 2 is odd (the rows of 32 threads start in different bank pairs); N rows still fit the
    // complex view.  Otherwise odd, read word by word.
    static constexpr int RP = N % 4 == 0 ? N + 2 : N + 1;
    static constexpr int floats = N * KP * 2;       // the complex plane is the larger of the two views
};

template <int N>
__global__ void __launch_bounds__(kXYThreads) k_fft_r2c_xy_reg(XYFwd P)
{
    typedef XYLayout<N> L;
    constexpr int H = L::H, NXH = L::NXH, KP = L::KP, RP = L::RP;
    __shared__ __attribute__((aligned(16))) float lds[L::floats];
    float2* cplane = reinterpret_cast<float2*>(lds);
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (P.planes < 0) lds[tid] = P.src[tid];        // never taken: tells the optimizer that LDS holds data
    const long plane = blockIdx.x;
    const long map = plane / P.sz;
    const int z = (int)(plane - map * P.sz);
    const float* src = P.src + plane * (long)P.sy * P.sx;
    float2* dst = P.dst + ((map * P.Nz + (long)z * P.tz + P.oz) * N) * NXH;

    // ---- the real rows into LDS, row y of the source at row y + oy, sample x at x + ox
    const bool padded = P.ox != 0 || P.sx != N;
    if (padded)
        for (int i = tid; i < P.sy * RP; i += kXYThreads) lds[P.oy * RP + i] = 0.f;
    __syncthreads();
    for (int r = wave; r < P.sy; r += kXYThreads / 64) {
#pragma unroll
        for (int c = 0; c * 64 < N; ++c) {
            const int s = c * 64 + lane - P.ox;
            if (c * 64 + lane < N && s >= 0 && s < P.sx)
                __builtin_amdgcn_global_load_lds((global_cptr)(src + (long)r * P.sx + s),
                                                 (lds_ptr)(lds + (r + P.oy) * RP + c * 64), 4, 0, 0);
        }
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    // ---- x: thread y transforms row y (rows outside the data are zero: nothing to do)
    const bool myrow = tid >= P.oy && tid < P.oy + P.sy;
    float2 X[NXH];
    if (myrow) {
        float2 x[H], y[H];
#pragma unroll
        for (int m = 0; m < H; ++m) {
            if constexpr (RP % 2 == 0) x[m] = *reinterpret_cast<const float2*>(lds + tid * RP + 2 * m);
            else x[m] = make_float2(lds[tid * RP + 2 * m], lds[tid * RP + 2 * m + 1]);
        }
        passes<H, -1, H, 1>(x, y);
        constexpr bool in_y = (count_passes(H) % 2) == 1;
        float2 (&Z)[H] = in_y ? y : x;
        X[0] = make_float2(Z[0].x + Z[0].y, 0.f);
        X[H] = make_float2(Z[0].x - Z[0].y, 0.f);
#pragma unroll
        for (int k = 1; k < H; ++k) {
            const float2 a = Z[k], b = Z[H - k];
            const float2 e = make_float2(a.x + b.x, a.y - b.y);
            const float2 d = make_float2(a.x - b.x, a.y + b.y);
            const float wc = TwTable<N>::t.c[k], ws = -TwTable<N>::t.s[k];
            X[k] = make_float2(0.5f * (e.x + wc * d.y + ws * d.x), 0.5f * (e.y + ws * d.y - wc * d.x));
        }
    }
    __syncthreads();                                // every row has been read: the complex view may overwrite it
    if (myrow) {
#pragma unroll
        for (int k = 0; k < NXH; ++k) cplane[tid * KP + k] = X[k];
    }
    __syncthreads();

    // ---- y: two threads per column (even extents), else thread k transforms column k; and stores it
    if constexpr (N % 2 == 0 && 2 * NXH <= kXYThreads) {
        const int c = tid >> 1, half = tid & 1;
        if (c < NXH) {
            constexpr int M = N / 2;
            float2 v[M], r[M];
#pragma unroll
            for (int m = 0; m < M; ++m) {
                const int e = 2 * m + half;
                v[m] = (e >= P.oy && e < P.oy + P.sy) ? cplane[e * KP + c] : make_float2(0.f, 0.f);
            }
            column_fft_by_lane_pair<N, -1>(v, r, half);
#pragma unroll
            for (int k = 0; k < M; ++k) dst[(long)(k + half * M) * NXH + c] = r[k];
        }
    } else if (tid < NXH) {
        float2 v[N], w[N];
#pragma unroll
        for (int e = 0; e < N; ++e)
            v[e] = (e >= P.oy && e < P.oy + P.sy) ? cplane[e * KP + tid] : make_float2(0.f, 0.f);
        passes<N, -1, N, 1>(v, w);
        constexpr bool in_w = (count_passes(N) % 2) == 1;
#pragma unroll
        for (int e = 0; e < N; ++e) dst[(long)e * NXH + tid] = in_w ? w[e] : v[e];
    }
}

template <int N>
__global__ void __launch_bounds__(kXYThreads, 2) k_fft_c2r_yx_reg(XYInv P)
{
    typedef XYLayout<N> L;
    constexpr int H = L::H, NXH = L::NXH, KP = L::KP, RP = L::RP;
    __shared__ __attribute__((aligned(16))) float lds[L::floats];
    float2* cplane = reinterpret_cast<float2*>(lds);
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const long plane = blockIdx.x;
    const long map = plane / P.dz;
    const int z = (int)(plane - map * P.dz);
    const float2* src = P.src + ((map * P.Nz + z + P.cz) * (long)N) * NXH;
    float* dst = P.dst + plane * (long)P.dy * P.dx;

    // ---- the spectrum plane into LDS as [y][k], row by row (coalesced, no registers on the way)
    if (P.planes < 0) lds[tid] = P.dst[tid];        // never taken: tells the optimizer that LDS holds data
    {
        const float* sf = reinterpret_cast<const float*>(src);
        for (int r = wave; r < N; r += kXYThreads / 64) {
#pragma unroll
            for (int c = 0; c * 64 < 2 * NXH; ++c) {
                if (c * 64 + lane < 2 * NXH)
                    __builtin_amdgcn_global_load_lds((global_cptr)(sf + (long)r * 2 * NXH + c * 64 + lane),
                                                     (lds_ptr)(lds + r * 2 * KP + c * 64), 4, 0, 0);
            }
        }
        __builtin_amdgcn_s_waitcnt(0);
    }
    __syncthreads();
    // ---- y: two threads per column (even extents), else thread k, invert column k in place
    if constexpr (N % 2 == 0 && 2 * NXH <= kXYThreads) {
        const int c = tid >> 1, half = tid & 1;
        if (c < NXH) {
            constexpr int M = N / 2;
            float2 v[M], r[M];
#pragma unroll
            for (int m = 0; m < M; ++m) v[m] = cplane[(2 * m + half) * KP + c];
            column_fft_by_lane_pair<N, +1>(v, r, half);
#pragma unroll
            for (int k = 0; k < M; ++k) cplane[(k + half * M) * KP + c] = r[k];
        }
    } else if (tid < NXH) {
        float2 v[N], w[N];
#pragma unroll
        for (int e = 0; e < N; ++e) v[e] = cplane[e * KP + tid];
        passes<N, +1, N, 1>(v, w);
        constexpr bool in_w = (count_passes(N) % 2) == 1;
#pragma unroll
        for (int e = 0; e < N; ++e) cplane[e * KP + tid] = in_w ? w[e] : v[e];
    }
    __syncthreads();

    // ---- x: thread y rebuilds the half-length spectrum of its row, inverts it and writes the real samples
    // over its own row (real rows keep the pitch of the complex rows, so no row touches another one's data)
    constexpr int RPI = 2 * KP;
    const int row = tid + P.cy;                     // thread t takes row t + cy of the plane, result row t
    if (tid < P.dy) {
        float2 x[H], y[H];
        {
            float2 X[NXH];
#pragma unroll
            for (int k = 0; k < NXH; ++k) X[k] = cplane[row * KP + k];
            x[0] = make_float2(X[0].x + X[H].x, X[0].x - X[H].x);
#pragma unroll
            for (int k = 1; k < H; ++k) {
                const float2 a = X[k], b = X[H - k];
                const float2 e = make_float2(a.x + b.x, a.y - b.y);
                const float2 d = make_float2(a.x - b.x, a.y + b.y);
                const float wc = TwTable<N>::t.c[k], ws = TwTable<N>::t.s[k];
                x[k] = make_float2(e.x - wc * d.y - ws * d.x, e.y + wc * d.x - ws * d.y);
            }
        }
        passes<H, +1, H, 1>(x, y);
        constexpr bool in_y = (count_passes(H) % 2) == 1;
        float2 (&zz)[H] = in_y ? y : x;
#pragma unroll
        for (int m = 0; m < H; ++m)
            cplane[row * KP + m] = make_float2(P.scale * zz[m].x, P.scale * zz[m].y);      // samples 2m, 2m+1
    }
    __syncthreads();
    for (int r = wave; r < P.dy; r += kXYThreads / 64) {
#pragma unroll
        for (int c = 0; c * 64 < N; ++c) {
            const int s = c * 64 + lane - P.cx;
            if (c * 64 + lane < N && s >= 0 && s < P.dx) dst[(long)r * P.dx + s] = lds[(r + P.cy) * RPI + c * 64 + lane];
        }
    }
}

// Forward x and y passes of planes that hold a few short rows (kernels: k_y rows of k_x taps), one wave per
// plane and NO LDS: lane k computes the coefficients X[r][k] of every source row directly from the taps
// (s_x real multiply-adds each; the taps are the same for all lanes and come through scalar loads) and
// then owns column k of the plane's spectrum: it runs the length-N transform along y in registers and
// stores the column.  The general kernel above spends a length-N/2 register transform per row on seven
// lanes and leaves its second wave idle during the y pass.
constexpr int kTapRows = 16, kTapCols = 16;

template <int N>
__global__ void __launch_bounds__(64) k_fft_r2c_xy_taps(XYFwd P)
{
    constexpr int NXH = N / 2 + 1;
    const int k = threadIdx.x;
    if (k >= NXH) return;
    const long plane = blockIdx.x;
    const long map = plane / P.sz;
    const int z = (int)(plane - map * P.sz);
    const float* src = P.src + plane * (long)P.sy * P.sx;       // uniform
    float2* dst = P.dst + ((map * P.Nz + (long)z * P.tz + P.oz) * N) * NXH;
    // exp(-2 pi i (x + ox) k / N) for the row's taps
    float2 tw[kTapCols];
#pragma unroll
    for (int x = 0; x < kTapCols; ++x) {
        const int m = ((x + P.ox) * k) % N;
        tw[x] = make_float2(TwTable<N>::t.c[m], -TwTable<N>::t.s[m]);
    }
    float2 v[N], w[N];
#pragma unroll
    for (int e = 0; e < N; ++e) v[e] = make_float2(0.f, 0.f);
#pragma unroll
    for (int r = 0; r < kTapRows; ++r) {
        if (r < P.sy) {     // uniform
            float2 a = make_float2(0.f, 0.f);
#pragma unroll
            for (int x = 0; x < kTapCols; ++x)
                if (x < P.sx) {     // uniform
                    const float t = src[r * P.sx + x];
                    a.x = fmaf(t, tw[x].x, a.x);
                    a.y = fmaf(t, tw[x].y, a.y);
                }
            v[r] = a;       // the launcher admits only planes whose rows start at y = 0
        }
    }
    passes<N, -1, N, 1>(v, w);
    constexpr bool in_w = (count_passes(N) % 2) == 1;
#pragma unroll
    for (int e = 0; e < N; ++e) dst[(long)e * NXH + k] = in_w ? w[e] : v[e];
}

template <int N>
int launch_xy(const XYFwd* F, const XYInv* B, hipStream_t s)
{
    const long planes = F ? F->planes : B->planes;
    if (planes >= 2147483647L) return fail(ZNN_EUNSUPPORTED, "too many planes for one launch");
    if (F && F->sy <= kTapRows && F->sx <= kTapCols && F->oy == 0 && kTapRows <= N && !tuning().fft_no_taps_pass) {
        ZNN_LAUNCH("fft r2c x and y of taps (registers)", s, (k_fft_r2c_xy_taps<N>), dim3((unsigned)planes), dim3(64), 0, *F);
        return check_launch("fused x/y pass of taps");
    }
    if (F) ZNN_LAUNCH("fft r2c x and y (registers)", s, (k_fft_r2c_xy_reg<N>), dim3((unsigned)planes), dim3(kXYThreads), 0, *F);
    else   ZNN_LAUNCH("fft c2r y and x (registers)", s, (k_fft_c2r_yx_reg<N>), dim3((unsigned)planes), dim3(kXYThreads), 0, *B);
    return check_launch("fused x/y pass");
}

}  // namespace

}  // namespace znn
