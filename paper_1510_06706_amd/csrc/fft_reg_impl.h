// Strided-axis FFT passes with the whole pencil in registers (templates; included by the
// fft_reg_*.hip translation units, which instantiate them for their share of the extents).
//
// The y and z passes of a 3D transform walk pencils whose elements are a row (or a plane)
// apart while NEIGHBOURING pencils are contiguous in memory.  One thread therefore owns one
// pencil: lane l of a wave loads element e of pencil p0 + l, the 64 loads of a wave are one
// contiguous run, and no LDS transpose is needed.  The transform itself is a Stockham
// autosort FFT (radices 4, 2, 3, 5) over a register array, fully unrolled: all indices and
// twiddle factors are compile-time constants, so a pass costs the butterfly arithmetic and
// nothing else (the LDS version spends most of its instructions on index arithmetic and LDS
// traffic and is bound by instruction issue, not by HBM).
//
// Instantiated for every 5-smooth extent from 8 to 96 (larger pencils do not fit the register file);
// everything else takes the LDS passes in fft.hip.  Rows known to be zero are not read
// (i0, ni) and rows outside the crop are not written (o0, no), as there.
#pragma once

#include "znn_internal.h"

namespace znn {

namespace {

constexpr int kThreads = 256;

// ---------------------------------------------------------------- compile-time twiddles
constexpr double kPi = 3.14159265358979323846264338327950288;

constexpr double series_sin(double x)
{
    const double x2 = x * x;
    double term = x, sum = x;
    for (int i = 1; i < 14; ++i) {
        term *= -x2 / ((2.0 * i) * (2.0 * i + 1.0));
        sum += term;
    }
    return sum;
}

constexpr double series_cos(double x)
{
    const double x2 = x * x;
    double term = 1.0, sum = 1.0;
    for (int i = 1; i < 14; ++i) {
        term *= -x2 / ((2.0 * i - 1.0) * (2.0 * i));
        sum += term;
    }
    return sum;
}

// cos and sin of 2 pi k / N, reduced to the first octant through the rational k / N.
template <int N>
struct Twiddles {
    float c[N], s[N];
    constexpr Twiddles() : c(), s()
    {
        for (int k = 0; k < N; ++k) {
            const int quad = (4 * k) / N;                       // quarter turn index 0..3
            const double frac = (double)(4 * k - quad * N) / (4.0 * N);     // in [0, 1/4)
            const double x = 2.0 * kPi * frac;                  // in [0, pi/2)
            double cc = 0.0, ss = 0.0;
            if (x <= kPi / 4) { cc = series_cos(x); ss = series_sin(x); }
            else { cc = series_sin(kPi / 2 - x); ss = series_cos(kPi / 2 - x); }
            double rc = cc, rs = ss;
            if (quad == 1) { rc = -ss; rs = cc; }
            else if (quad == 2) { rc = -cc; rs = -ss; }
            else if (quad == 3) { rc = ss; rs = -cc; }
            c[k] = (float)rc;
            s[k] = (float)rs;
        }
    }
};

template <int N> struct TwTable { static constexpr Twiddles<N> t = Twiddles<N>(); };

__device__ __forceinline__ float2 cadd(float2 a, float2 b) { return make_float2(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ float2 csub(float2 a, float2 b) { return make_float2(a.x - b.x, a.y - b.y); }
template <int DIR> __device__ __forceinline__ float2 mul_di(float2 a)   // times DIR * i
{
    return DIR > 0 ? make_float2(-a.y, a.x) : make_float2(a.y, -a.x);
}

// a * exp(DIR 2 pi i K / N) with K a compile-time constant
template <int N, int DIR, int K>
__device__ __forceinline__ float2 twmul(float2 a)
{
    constexpr int k = ((K % N) + N) % N;
    if constexpr (k == 0) return a;
    else if constexpr (4 * k == N) return mul_di<DIR>(a);
    else if constexpr (2 * k == N) return make_float2(-a.x, -a.y);
    else if constexpr (4 * k == 3 * N) return mul_di<-DIR>(a);
    else {
        constexpr float c = TwTable<N>::t.c[k];
        constexpr float s = DIR > 0 ? TwTable<N>::t.s[k] : -TwTable<N>::t.s[k];
        return make_float2(a.x * c - a.y * s, a.x * s + a.y * c);
    }
}

constexpr int pick_radix(int n) { return n % 4 == 0 ? 4 : n % 2 == 0 ? 2 : n % 3 == 0 ? 3 : 5; }

// One butterfly of a Stockham pass: inputs x[q + S (PP + M j)], outputs y[q + S (R PP + j)],
// output j multiplied by exp(DIR 2 pi i j PP S / N).
template <int N, int DIR, int R, int M, int S, int PP, int Q>
__device__ __forceinline__ void butterfly(const float2 (&x)[N], float2 (&y)[N])
{
    constexpr int xi = Q + S * PP, xs = S * M;
    constexpr int yi = Q + S * R * PP, ys = S;
    constexpr int ti = PP * S;
    if constexpr (R == 4) {
        const float2 a0 = x[xi], a1 = x[xi + xs], a2 = x[xi + 2 * xs], a3 = x[xi + 3 * xs];
        const float2 s02 = cadd(a0, a2), d02 = csub(a0, a2);
        const float2 s13 = cadd(a1, a3), d13 = mul_di<DIR>(csub(a1, a3));
        y[yi] = cadd(s02, s13);
        y[yi + ys] = twmul<N, DIR, ti>(cadd(d02, d13));
        y[yi + 2 * ys] = twmul<N, DIR, 2 * ti>(csub(s02, s13));
        y[yi + 3 * ys] = twmul<N, DIR, 3 * ti>(csub(d02, d13));
    } else if constexpr (R == 2) {
        const float2 a0 = x[xi], a1 = x[xi + xs];
        y[yi] = cadd(a0, a1);
        y[yi + ys] = twmul<N, DIR, ti>(csub(a0, a1));
    } else if constexpr (R == 3) {
        const float2 a0 = x[xi], a1 = x[xi + xs], a2 = x[xi + 2 * xs];
        const float2 t1 = cadd(a1, a2);
        const float2 t2 = make_float2(a0.x - 0.5f * t1.x, a0.y - 0.5f * t1.y);
        float2 t3 = csub(a1, a2);
        t3 = mul_di<DIR>(make_float2(0.8660254037844386f * t3.x, 0.8660254037844386f * t3.y));
        y[yi] = cadd(a0, t1);
        y[yi + ys] = twmul<N, DIR, ti>(cadd(t2, t3));
        y[yi + 2 * ys] = twmul<N, DIR, 2 * ti>(csub(t2, t3));
    } else {
        constexpr float c1 = 0.30901699437494745f, c2 = -0.8090169943749475f;
        constexpr float s1 = 0.9510565162951535f, s2 = 0.5877852522924731f;
        const float2 a0 = x[xi], a1 = x[xi + xs], a2 = x[xi + 2 * xs], a3 = x[xi + 3 * xs], a4 = x[xi + 4 * xs];
        const float2 t1 = cadd(a1, a4), t2 = cadd(a2, a3), t3 = csub(a1, a4), t4 = csub(a2, a3);
        const float2 m1 = make_float2(a0.x + c1 * t1.x + c2 * t2.x, a0.y + c1 * t1.y + c2 * t2.y);
        const float2 m2 = make_float2(a0.x + c2 * t1.x + c1 * t2.x, a0.y + c2 * t1.y + c1 * t2.y);
        const float2 n1 = mul_di<DIR>(make_float2(s1 * t3.x + s2 * t4.x, s1 * t3.y + s2 * t4.y));
        const float2 n2 = mul_di<DIR>(make_float2(s2 * t3.x - s1 * t4.x, s2 * t3.y - s1 * t4.y));
        y[yi] = cadd(a0, cadd(t1, t2));
        y[yi + ys] = twmul<N, DIR, ti>(cadd(m1, n1));
        y[yi + 2 * ys] = twmul<N, DIR, 2 * ti>(cadd(m2, n2));
        y[yi + 3 * ys] = twmul<N, DIR, 3 * ti>(csub(m2, n2));
        y[yi + 4 * ys] = twmul<N, DIR, 4 * ti>(csub(m1, n1));
    }
}

// All butterflies of one pass: U runs over the M * S pairs (PP, Q).
template <int N, int DIR, int R, int M, int S, int U>
__device__ __forceinline__ void pass_units(const float2 (&x)[N], float2 (&y)[N])
{
    if constexpr (U < M * S) {
        butterfly<N, DIR, R, M, S, U / S, U % S>(x, y);
        pass_units<N, DIR, R, M, S, U + 1>(x, y);
    }
}

// Stockham passes from length n (stride s = N / n) down to 1; the result lands in `x`
// when the number of remaining passes is even and in `y` when it is odd.
template <int N, int DIR, int n, int s>
__device__ __forceinline__ void passes(float2 (&x)[N], float2 (&y)[N])
{
    if constexpr (n > 1) {
        constexpr int r = pick_radix(n);
        pass_units<N, DIR, r, n / r, s, 0>(x, y);
        passes<N, DIR, n / r, s * r>(y, x);
    }
}

constexpr int count_passes(int n) { int c = 0; while (n > 1) { n /= pick_radix(n); ++c; } return c; }

// the value that the other lane of the pair (lane ^ 1) holds: a DPP move within the quad, no LDS
__device__ __forceinline__ float from_pair_lane(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, false));
}

// z[k] *= exp(DIR 2 pi i k / N) for k < M on the lanes with `odd` set (the constants are compile-time)
template <int N, int DIR, int M, int K = 0>
__device__ __forceinline__ void static_for_twiddle(float2 (&z)[M], int odd)
{
    if constexpr (K < M) {
        const float2 t = twmul<N, DIR, K>(z[K]);
        if (odd) z[K] = t;
        static_for_twiddle<N, DIR, M, K + 1>(z, odd);
    }
}

// Length-N transform (N even) of a column by TWO neighbouring lanes: lane `half` of the pair holds the
// samples 2 m + half in v[m], transforms them (length N/2), the odd lane multiplies its results by the
// twiddles exp(DIR 2 pi i k / N), the lanes swap results, and the even lane ends up with the coefficients
// k = 0 .. N/2 - 1, the odd lane with N/2 .. N - 1, in r[].  Two thirds of the instructions of the length-N
// transform on one lane, and the column pass occupies both waves of the workgroup instead of 49 lanes of one.
template <int N, int DIR>
__device__ __forceinline__ void column_fft_by_lane_pair(float2 (&v)[N / 2], float2 (&r)[N / 2], int half)
{
    constexpr int M = N / 2;
    float2 w[M];
    passes<M, DIR, M, 1>(v, w);
    constexpr bool in_w = (count_passes(M) % 2) == 1;
    float2 (&z)[M] = in_w ? w : v;
    static_for_twiddle<N, DIR, M>(z, half);
#pragma unroll
    for (int k = 0; k < M; ++k) {
        // the partner's value of the same k
        const float2 o = make_float2(from_pair_lane(z[k].x), from_pair_lane(z[k].y));
        r[k] = half ? csub(o, z[k]) : cadd(z[k], o);
    }
}

template <int N, int DIR>
__global__ void __launch_bounds__(kThreads)
k_fft_axis_reg(RegAxis P)
{
    if constexpr (N % 2 == 0) {
        // two neighbouring lanes per pencil: half the registers per lane (a length-96 pencil held by one lane
        // takes the whole register file of a SIMD for one wave) and two thirds of the instructions
        constexpr int M = N / 2;
        const unsigned g2 = blockIdx.x * kThreads + threadIdx.x;
        const unsigned g = g2 >> 1;
        const int half = (int)(g2 & 1);
        if (g >= (unsigned)P.Ob * (unsigned)P.L) return;
        const unsigned ob = fdiv(g, P.fL);
        const unsigned l = g - ob * (unsigned)P.L;
        const long oa = blockIdx.y;
        const float2* in = P.in + oa * P.in_sa + (long)ob * P.in_sb + l;
        float2* out = P.out + oa * P.out_sa + (long)ob * P.out_sb + l;
        float2 v[M], r[M];
#pragma unroll
        for (int m = 0; m < M; ++m) {
            const int e = 2 * m + half;
            v[m] = (e >= P.i0 && e < P.i0 + P.ni) ? in[(long)e * P.stride] : make_float2(0.f, 0.f);
        }
        column_fft_by_lane_pair<N, DIR>(v, r, half);
#pragma unroll
        for (int k = 0; k < M; ++k) {
            const int e = k + half * M;
            if (e >= P.o0 && e < P.o0 + P.no) out[(long)e * P.stride] = r[k];
        }
    } else {
        const unsigned g = blockIdx.x * kThreads + threadIdx.x;
        if (g >= (unsigned)P.Ob * (unsigned)P.L) return;
        const unsigned ob = fdiv(g, P.fL);
        const unsigned l = g - ob * (unsigned)P.L;
        const long oa = blockIdx.y;
        const float2* in = P.in + oa * P.in_sa + (long)ob * P.in_sb + l;
        float2* out = P.out + oa * P.out_sa + (long)ob * P.out_sb + l;
        float2 x[N], y[N];
#pragma unroll
        for (int e = 0; e < N; ++e)
            x[e] = (e >= P.i0 && e < P.i0 + P.ni) ? in[(long)e * P.stride] : make_float2(0.f, 0.f);
        passes<N, DIR, N, 1>(x, y);
        constexpr bool in_y = (count_passes(N) % 2) == 1;
#pragma unroll
        for (int e = 0; e < N; ++e)
            if (e >= P.o0 && e < P.o0 + P.no) out[(long)e * P.stride] = in_y ? y[e] : x[e];
    }
}

template <int N>
int launch_n(const RegAxis& P, int dir, hipStream_t s)
{
    const long threads = (long)P.Ob * P.L * (N % 2 == 0 ? 2 : 1);      // even lengths: two lanes per pencil
    const dim3 grid((unsigned)((threads + kThreads - 1) / kThreads), (unsigned)P.Oa);
    if (dir > 0) ZNN_LAUNCH("fft axis inverse (registers)", s, (k_fft_axis_reg<N, +1>), grid, dim3(kThreads), 0, P);
    else         ZNN_LAUNCH("fft axis forward (registers)", s, (k_fft_axis_reg<N, -1>), grid, dim3(kThreads), 0, P);
    return check_launch("register FFT pass");
}

}  // namespace

}  // namespace znn
