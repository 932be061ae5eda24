// Per-frequency multiply-accumulate of the FFT method (Section 4) with the last axis of
// the kernel transform folded in.
//
// A kernel has only KZ non-zero planes along its slowest axis, so its full spectrum is
// N / KZ times larger than the information in it, and streaming the full spectra of all
// f*f' kernels is what bounds the plain multiply-accumulate (HBM).  Here the kernels are
// transformed along the fast axes only ("half spectra", [pair][a][P], a < KZ, P = elements
// per plane), and the sum over the taps,
//     W^[wz] = sum_a Wh[a] exp(-2 pi i a wz / N),
// is evaluated in registers right before the product with the node spectrum.  Kernel
// traffic drops by N / KZ and the kernel becomes ALU-bound.
//
// A thread owns one in-plane frequency p and 4*Z0 frequencies along the axis, chosen a
// quarter period apart: wz = z0 + q N/4, q = 0..3.  For those,
//     W^[z0 + q N/4] = sum_a (Wh[a] t_a(z0)) (-i)^(a q),   t_a(z0) = exp(-2 pi i a z0 / N),
// so after KZ-1 complex multiplications by twiddles that stay in registers the four
// frequencies cost a radix-4 butterfly of additions (taps with equal a mod 4 are folded
// first).  Every thread walks the reduction index (input nodes forward, output nodes
// backward) for G result nodes, so a loaded node-spectrum value is used G times and a
// loaded half-spectrum value 4*Z0 times.  A wave owns 64 neighbouring p: its loads and
// stores are contiguous runs of one plane row.
//
// Needs N divisible by 4 and taps one voxel apart along the axis; other layers use the
// full-spectrum multiply-accumulate.
#include "znn_internal.h"

namespace znn {

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float2 cmulf(float2 a, float2 b)
{
    return make_float2(fmaf(a.x, b.x, -a.y * b.y), fmaf(a.x, b.y, a.y * b.x));
}

// Grid order.  A workgroup is `wpb` waves that share 64 in-plane frequencies and differ in
// their frequencies along the folded axis: all of them request the same half-spectrum lines,
// which then come out of the compute unit's cache instead of `wpb` times out of L2/HBM.
// Workgroups that differ only in their group of result nodes read the same node spectra X;
// the hardware deals consecutive workgroups to the eight XCDs (each with its own L2) in turn,
// so the flat workgroup index is taken apart as
//     xcd = b % 8,  slot = b / 8,  frequency block q = (slot / ngroups) * 8 + xcd,
//     node group = slot % ngroups:
// the workgroups of one frequency block run on one XCD, next to each other in time, and X
// comes out of that XCD's L2 for all but the first of them (config 5: 20 GB fetched from
// HBM per launch before, where the algorithm reads 4.2 GB).
template <bool BWD, int KZ, int Z0, int G>
__global__ void __launch_bounds__(kThreads)
k_mac_fused(int f, int fo, int N, int P, int nzi, int wpb, int nq, int ngroups, const float2* __restrict__ Wh,
            const float2* __restrict__ X, float2* __restrict__ Y)
{
    const int npc = (P + 63) >> 6;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int q = (slot / ngroups) * 8 + xcd, og = slot % ngroups;
    if (q >= nq) return;
    const int pc = q % npc, zb = q / npc;
    const int zi = zb * wpb + (threadIdx.x >> 6);
    const int p = pc * 64 + (threadIdx.x & 63);
    if (zi >= nzi || p >= P) return;
    const int o0 = og * G;
    const int nred = BWD ? fo : f, nout = BWD ? f : fo;
    const int Q = N >> 2;
    const long vol = (long)N * P;

    float2 tw[Z0][KZ > 1 ? KZ - 1 : 1];
#pragma unroll
    for (int m = 0; m < Z0; ++m) {
        const int z0 = zi * Z0 + m;
#pragma unroll
        for (int a = 1; a < KZ; ++a) {
            const int idx = (a * z0) % N;
            float sn, cs;
            sincospif(2.0f * (float)idx / (float)N, &sn, &cs);
            tw[m][a - 1] = make_float2(cs, -sn);
        }
    }
    float2 acc[G][Z0][4];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int m = 0; m < Z0; ++m)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[g][m][q] = make_float2(0.f, 0.f);

    const float2* xbase = X + (long)(zi * Z0) * P + p;
    const long wplane = (long)KZ * P;
    for (int r = 0; r < nred; ++r) {
        float2 x[Z0][4];
#pragma unroll
        for (int m = 0; m < Z0; ++m)
#pragma unroll
            for (int q = 0; q < 4; ++q) x[m][q] = xbase[(long)r * vol + (long)(m + q * Q) * P];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const int o = min(o0 + g, nout - 1);
            const long pair = BWD ? (long)r * f + o : (long)o * f + r;     // kernels are [f'][f]
            const float2* wp = Wh + pair * wplane + p;
            float2 w[KZ];
#pragma unroll
            for (int a = 0; a < KZ; ++a) w[a] = wp[(long)a * P];
#pragma unroll
            for (int m = 0; m < Z0; ++m) {
                // fold the rotated taps by a mod 4
                float2 v[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) v[c] = make_float2(0.f, 0.f);
#pragma unroll
                for (int a = 0; a < KZ; ++a) {
                    const float2 u = a == 0 ? w[0] : cmulf(w[a], tw[m][a - 1]);
                    v[a & 3].x += u.x;
                    v[a & 3].y += u.y;
                }
                // radix-4 butterfly: W^_q = sum_c v_c (-i)^(c q)
                const float2 s02 = make_float2(v[0].x + v[2].x, v[0].y + v[2].y);
                const float2 d02 = make_float2(v[0].x - v[2].x, v[0].y - v[2].y);
                const float2 s13 = make_float2(v[1].x + v[3].x, v[1].y + v[3].y);
                const float2 d13 = make_float2(v[1].x - v[3].x, v[1].y - v[3].y);
                float2 wq[4];
                wq[0] = make_float2(s02.x + s13.x, s02.y + s13.y);
                wq[2] = make_float2(s02.x - s13.x, s02.y - s13.y);
                wq[1] = make_float2(d02.x + d13.y, d02.y - d13.x);      // d02 - i d13
                wq[3] = make_float2(d02.x - d13.y, d02.y + d13.x);      // d02 + i d13
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float2 xv = x[m][q];
                    if (BWD) {      // conj(W^) x
                        acc[g][m][q].x = fmaf(wq[q].x, xv.x, fmaf(wq[q].y, xv.y, acc[g][m][q].x));
                        acc[g][m][q].y = fmaf(wq[q].x, xv.y, fmaf(-wq[q].y, xv.x, acc[g][m][q].y));
                    } else {
                        acc[g][m][q].x = fmaf(wq[q].x, xv.x, fmaf(-wq[q].y, xv.y, acc[g][m][q].x));
                        acc[g][m][q].y = fmaf(wq[q].x, xv.y, fmaf(wq[q].y, xv.x, acc[g][m][q].y));
                    }
                }
            }
        }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
        if (o0 + g >= nout) break;
        float2* yp = Y + (long)(o0 + g) * vol + (long)(zi * Z0) * P + p;
#pragma unroll
        for (int m = 0; m < Z0; ++m)
#pragma unroll
            for (int q = 0; q < 4; ++q) yp[(long)(m + q * Q) * P] = acc[g][m][q];
    }
}

template <bool BWD, int KZ, int Z0>
int launch_variant(int f, int fo, int N, int P, const float2* Wh, const float2* X, float2* Y, hipStream_t s)
{
    constexpr int G = fft_mac_group(Z0);
    const int nout = BWD ? f : fo;
    const int nzi = N / 4 / Z0;
    // waves per workgroup: four, or three when that splits the frequency groups evenly (N = 96: 6 = 3 + 3)
    const int wpb = nzi % 4 != 0 && nzi % 3 == 0 ? 3 : 4;
    const long nq = (long)((P + 63) / 64) * ((nzi + wpb - 1) / wpb);
    const int ngroups = (nout + G - 1) / G;
    const long blocks = ((nq + 7) / 8) * 8 * ngroups;
    if (blocks >= 2147483647L) return fail(ZNN_EUNSUPPORTED, "too many frequencies");
    ZNN_LAUNCH(BWD ? "spectral mac backward (taps folded in)" : "spectral mac forward (taps folded in)", s,
               (k_mac_fused<BWD, KZ, Z0, G>), dim3((unsigned)blocks), dim3(64 * wpb), 0, f, fo, N, P, nzi, wpb,
               (int)nq, ngroups, Wh, X, Y);
    return check_launch("spectral multiply-accumulate");
}

template <bool BWD, int KZ>
int launch_kz(int z0, int f, int fo, int N, int P, const float2* Wh, const float2* X, float2* Y, hipStream_t s)
{
    if (z0 == 4) return launch_variant<BWD, KZ, 4>(f, fo, N, P, Wh, X, Y, s);
    if (z0 == 2) return launch_variant<BWD, KZ, 2>(f, fo, N, P, Wh, X, Y, s);
    return launch_variant<BWD, KZ, 1>(f, fo, N, P, Wh, X, Y, s);
}

template <bool BWD>
int launch_dir(int taps, int z0, int f, int fo, int N, int P, const float2* Wh, const float2* X, float2* Y, hipStream_t s)
{
    switch (taps) {
        case 1: return launch_kz<BWD, 1>(z0, f, fo, N, P, Wh, X, Y, s);
        case 2: return launch_kz<BWD, 2>(z0, f, fo, N, P, Wh, X, Y, s);
        case 3: return launch_kz<BWD, 3>(z0, f, fo, N, P, Wh, X, Y, s);
        case 4: return launch_kz<BWD, 4>(z0, f, fo, N, P, Wh, X, Y, s);
        case 5: return launch_kz<BWD, 5>(z0, f, fo, N, P, Wh, X, Y, s);
        case 6: return launch_kz<BWD, 6>(z0, f, fo, N, P, Wh, X, Y, s);
        case 7: return launch_kz<BWD, 7>(z0, f, fo, N, P, Wh, X, Y, s);
        case 8: return launch_kz<BWD, 8>(z0, f, fo, N, P, Wh, X, Y, s);
        case 9: return launch_kz<BWD, 9>(z0, f, fo, N, P, Wh, X, Y, s);
        case 10: return launch_kz<BWD, 10>(z0, f, fo, N, P, Wh, X, Y, s);
        case 11: return launch_kz<BWD, 11>(z0, f, fo, N, P, Wh, X, Y, s);
        case 12: return launch_kz<BWD, 12>(z0, f, fo, N, P, Wh, X, Y, s);
        case 13: return launch_kz<BWD, 13>(z0, f, fo, N, P, Wh, X, Y, s);
        case 14: return launch_kz<BWD, 14>(z0, f, fo, N, P, Wh, X, Y, s);
        case 15: return launch_kz<BWD, 15>(z0, f, fo, N, P, Wh, X, Y, s);
        case 16: return launch_kz<BWD, 16>(z0, f, fo, N, P, Wh, X, Y, s);
        default: return fail(ZNN_EUNSUPPORTED, "more taps than the folded multiply-accumulate takes");
    }
}

}  // namespace

int fft_mac_fused(bool backward, int taps, int z0, int f, int fo, int N, int P, const float2* Wh,
                  const float2* X, float2* Y, hipStream_t s)
{
    if (N % 4 != 0 || taps < 1 || taps > kMaxFoldedTaps || (z0 != 1 && z0 != 2 && z0 != 4) || (N / 4) % z0 != 0)
        return fail(ZNN_EUNSUPPORTED, "layer does not fit the folded multiply-accumulate");
    return backward ? launch_dir<true>(taps, z0, f, fo, N, P, Wh, X, Y, s)
                    : launch_dir<false>(taps, z0, f, fo, N, P, Wh, X, Y, s);
}

}  // namespace znn
