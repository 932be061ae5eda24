// Strided-axis FFT passes for pencils too long for one thread's registers (N > 96), in two levels.
//
// N = N1 * N2 with N1, N2 <= 16.  With n = n1 + N1 n2 and k = N2 k1 + k2,
//   X[N2 k1 + k2] = sum_n1 w_N1^(n1 k1) w_N^(n1 k2) [ sum_n2 x[n1 + N1 n2] w_N2^(n2 k2) ],
// so a thread keeps N2 samples of a pencil in registers at the first level and N1 at the second (the
// unrolled register transforms of fft_reg_impl.h), the pencil makes ONE trip through LDS and the workgroup
// meets at ONE barrier after its loads.  (The radix passes in fft.hip: load, one pass per radix, store, a
// barrier between each, every element through LDS once per pass.)  A workgroup takes 16 neighbouring pencils
// (128 contiguous bytes per element row): thread (n1, pencil) loads its samples straight from global memory,
// transforms over n2, multiplies by w_N^(n1 k2) and parks the result in LDS; thread (k2, pencil) then
// transforms over n1 and stores.  Inputs known to be zero are not read, outputs outside the crop not written.
// Measured on the 2D benchmark layer (N = 256): 33 -> 20 us per pass.
#include "fft_reg_impl.h"

namespace znn {

namespace {

constexpr int kPencils = 16, kPitch = 17;

template <int M, int DIR>
__device__ __forceinline__ void small_fft(float2 (&v)[M])
{
    float2 w[M];
    passes<M, DIR, M, 1>(v, w);
    if constexpr ((count_passes(M) % 2) == 1) {
#pragma unroll
        for (int e = 0; e < M; ++e) v[e] = w[e];
    }
}

template <int N1, int N2, int DIR>
__global__ void __launch_bounds__(kPencils * (N1 > N2 ? N1 : N2)) k_fft_axis_two_level(TwoLevelAxis P)
{
    constexpr int N = N1 * N2, R = N1 > N2 ? N1 : N2;
    __shared__ float2 buf[N * kPitch];
    __shared__ float2 tw[N];
    for (int t = threadIdx.x; t < N; t += kPencils * R) {
        float sn, cs;
        sincospif(2.0f * (float)t / (float)N, &sn, &cs);
        tw[t] = make_float2(cs, DIR > 0 ? sn : -sn);
    }
    // the launcher keeps the grid below 2^32 / (largest divisor), so these are exact
    const unsigned blk = blockIdx.x;
    unsigned o = fdiv(blk, P.fchunks);
    const int chunk = (int)(blk - o * P.chunks);
    const unsigned o2 = fdiv(o, P.foc);
    const int oc = (int)(o - o2 * P.Oc);
    const int oa = (int)fdiv(o2, P.fob);
    const int ob = (int)(o2 - (unsigned)oa * P.Ob);
    const int p0 = chunk * kPencils;
    const int p = threadIdx.x & 15, hi = threadIdx.x >> 4;     // pencil of the chunk; n1 at the first level, k2 at the second
    const bool live = p0 + p < P.L;
    const float2* in = P.in + (oa * P.in_sa + ob * P.in_sb + oc * P.in_sc) + p0 + p;
    float2 v[N2];
    if (hi < N1) {
#pragma unroll
        for (int n2 = 0; n2 < N2; ++n2) {
            const int e = hi + N1 * n2;
            v[n2] = (live && e >= P.i0 && e < P.i0 + P.ni) ? in[e * P.in_stride] : make_float2(0.f, 0.f);
        }
        small_fft<N2, DIR>(v);
    }
    __syncthreads();        // the twiddles are in place
    if (hi < N1) {
#pragma unroll
        for (int k2 = 0; k2 < N2; ++k2) {
            const float2 w = tw[hi * k2];       // n1 k2 < N
            const float2 t = k2 == 0 ? v[0] : make_float2(v[k2].x * w.x - v[k2].y * w.y, v[k2].x * w.y + v[k2].y * w.x);
            buf[(hi * N2 + k2) * kPitch + p] = t;
        }
    }
    __syncthreads();
    if (hi < N2) {
        float2 u[N1];
#pragma unroll
        for (int n1 = 0; n1 < N1; ++n1) u[n1] = buf[(n1 * N2 + hi) * kPitch + p];
        small_fft<N1, DIR>(u);
        float2* out = P.out + (oa * P.out_sa + ob * P.out_sb + oc * P.out_sc) + p0 + p;
        if (live) {
#pragma unroll
            for (int k1 = 0; k1 < N1; ++k1) {
                const int k = N2 * k1 + hi;
                if (k >= P.o0 && k < P.o0 + P.no) out[k * P.out_stride] = u[k1];
            }
        }
    }
}

template <int N1, int N2>
int launch_two_level(const TwoLevelAxis& P, long blocks, int dir, hipStream_t s)
{
    constexpr int threads = kPencils * (N1 > N2 ? N1 : N2);
    if (dir > 0) ZNN_LAUNCH("fft axis inverse (two levels)", s, (k_fft_axis_two_level<N1, N2, +1>), dim3((unsigned)blocks), dim3(threads), 0, P);
    else         ZNN_LAUNCH("fft axis forward (two levels)", s, (k_fft_axis_two_level<N1, N2, -1>), dim3((unsigned)blocks), dim3(threads), 0, P);
    return check_launch("two-level FFT pass");
}

}  // namespace

// Every 5-smooth length from 100 to 256 that is a product of two factors of at most 16.
bool fft_axis_two_level_supported(int N)
{
    switch (N) {
        case 100: case 108: case 120: case 128: case 135: case 144: case 150: case 160: case 180: case 192:
        case 225: case 240: case 256: return true;
    }
    return false;
}

int fft_axis_two_level(TwoLevelAxis P, int dir, hipStream_t s)
{
    const int chunks = (P.L + kPencils - 1) / kPencils;
    P.chunks = chunks;
    P.fchunks = make_fastdiv((unsigned)chunks);
    P.foc = make_fastdiv((unsigned)P.Oc);
    P.fob = make_fastdiv((unsigned)P.Ob);
    const long blocks = (long)P.Oa * P.Ob * P.Oc * chunks;
    long dmax = chunks;
    if (P.Oc > dmax) dmax = P.Oc;
    if (P.Ob > dmax) dmax = P.Ob;
    if (blocks * dmax >= 4294967296L) return fail(ZNN_EUNSUPPORTED, "too many pencils for one launch");
    switch (P.N) {
        case 100: return launch_two_level<10, 10>(P, blocks, dir, s);
        case 108: return launch_two_level<12, 9>(P, blocks, dir, s);
        case 120: return launch_two_level<12, 10>(P, blocks, dir, s);
        case 128: return launch_two_level<16, 8>(P, blocks, dir, s);
        case 135: return launch_two_level<15, 9>(P, blocks, dir, s);
        case 144: return launch_two_level<12, 12>(P, blocks, dir, s);
        case 150: return launch_two_level<15, 10>(P, blocks, dir, s);
        case 160: return launch_two_level<16, 10>(P, blocks, dir, s);
        case 180: return launch_two_level<15, 12>(P, blocks, dir, s);
        case 192: return launch_two_level<16, 12>(P, blocks, dir, s);
        case 225: return launch_two_level<15, 15>(P, blocks, dir, s);
        case 240: return launch_two_level<16, 15>(P, blocks, dir, s);
        case 256: return launch_two_level<16, 16>(P, blocks, dir, s);
    }
    return fail(ZNN_EUNSUPPORTED, "no two-level pass for extent %d", P.N);
}

}  // namespace znn
