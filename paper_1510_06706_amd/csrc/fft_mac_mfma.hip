// Per-frequency multiply-accumulate of the FFT method (Section 4) with the last axis of the
// kernel transform folded in, the rebuild of the kernel spectrum on the matrix cores.
//
// The folded multiply-accumulate (fft_mac.hip) is bound by vector-ALU instruction issue: per
// edge and frequency it spends about three times as many instructions on rebuilding
//     W^[w] = sum_a Wh[a] exp(-2 pi i a w / N)
// from the half spectrum Wh as on the product with the node spectrum.  That rebuild is a small
// dense matrix product with a constant matrix of twiddles, so here it runs on the otherwise
// idle fp32 matrix cores, and the vector ALUs keep only what is per frequency.
//
// With w = z0 + q N/4 (q = 0..3),
//     W^[z0 + q N/4] = sum_c V_c[z0] (-i)^(c q),   V_c[z0] = sum_{a = c mod 4} Wh[a] exp(-2 pi i a z0 / N),
// so only the four class sums V_c are matrix products (over the two to four taps of a class);
// the four frequencies then follow from a radix-4 butterfly of additions.
//
//   D[m][n] += A[m][k] * B[k][n]                  v_mfma_f32_16x16x4_f32
//     m : (z0 in a group of 8, re | im)            A = twiddles, constant, in registers
//     n : 16 neighbouring in-plane frequencies p   B = half-spectrum values, straight from global memory
//     k : (tap of the class, re | im)
// The accumulator layout gives lane (g, n) the complete complex numbers V_c[8t + 2g + e], e = 0, 1,
// of all four classes at its p = p0 + n: butterfly and product need no exchange between lanes.
//
// A wave owns 16 p, ZG groups of 8 z0 (= 32 ZG frequencies along the folded axis) and G result
// nodes; it walks the reduction index (input nodes forward, output nodes backward).  The four
// waves of a workgroup share the node-spectrum tile of the current reduction index through LDS
// (two buffers taking turns), so a tile is fetched once for 4 G result nodes.  Workgroups that
// differ only in their result nodes run next to each other on one XCD (see fft_mac.hip).
//
// Where a wave owns the whole folded axis (N = 32 ZG) the kernel can also apply the inverse transform
// along that axis to its sums before it stores them, which saves the separate pass over the result
// spectra: with z = q N/4 + z0 and m = m0 + 4 m1,
//     y[m0 + 4 m1] = sum_z0 exp(+2 pi i z0 m1 / (N/4)) * exp(+2 pi i z0 m0 / N) * sum_q Y[q N/4 + z0] i^(q m0),
// i.e. a radix-4 butterfly over the four values a lane already holds per z0, a twiddle, and N/4-point
// transforms over z0, for which the lanes exchange their values through a wave-private piece of LDS.
//
// Needs N divisible by 32 and taps one voxel apart; other layers use the vector-ALU kernel.
#include "znn_internal.h"
#include "fft_reg_impl.h"       // passes<>: the register FFT of the strided-axis kernels

namespace znn {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) const void* global_cptr;
typedef __attribute__((address_space(3))) void* lds_ptr;

constexpr int kWaves = 4;
constexpr int kG = 2;                   // result nodes per wave
constexpr int kTileMax = 3 * 32 * 16;   // ZG <= 3 groups of 8 z0, four quarter-period blocks, 16 p

// taps of class c (a = c, c + 4, ...) and the MFMA k-steps they take (two rows per tap, four per step)
constexpr int class_taps(int KZ, int c) { return c < KZ ? (KZ - c + 3) / 4 : 0; }
constexpr int class_steps(int KZ, int c) { return (2 * class_taps(KZ, c) + 3) / 4; }
constexpr int steps_before(int KZ, int c) { return c == 0 ? 0 : steps_before(KZ, c - 1) + class_steps(KZ, c - 1); }
constexpr int total_steps(int KZ) { return steps_before(KZ, 4); }

struct MacTile {
    const float2* Wh;       // half spectra [pair][KZ][P]
    const float2* X;        // node spectra read   [nred][N][P]
    float2* Y;              // node spectra written [nout][N][P]
    int f, fo, N, P;
    int nslice;             // slices of ZG z0-groups along the folded axis (N / 32 / ZG); a workgroup takes one
    int nq;                 // p tiles * slices
    int ngroups;            // groups of 4 G result nodes (G per wave)
    int zinv_o0, zinv_no;   // zinv_no > 0: store the inverse transform along the folded axis, rows [o0, o0 + no) only
};

// ZINV: the sums are stored transformed back along the folded axis (rows [zinv_o0, zinv_o0 + zinv_no)); the
// host asks for it only where a wave owns the whole axis, N = 32 ZG
// (three waves per SIMD asked for where the loop fits them: the transform at the end would otherwise be
// given a few registers more than the loop needs and cost the kernel a wave)
template <bool BWD, int KZ, int ZG, bool ZINV>
__global__ void __launch_bounds__(64 * kWaves, (ZG <= 2 && KZ <= 8) ? 3 : 2) k_mac_mfma(MacTile T)
{
    constexpr int G = kG;
    constexpr int NB = total_steps(KZ);
    // Two node-spectrum tiles (ZG * 32 rows x 16 p each) as two
    // separate LDS objects: the compiler then knows that the loads landing in one do not alias the
    // reads of the other and does not wait for them before those reads.
    __shared__ float2 tileA[kTileMax], tileB[kTileMax];
    // for the inverse transform of the sums: per wave two blocks of N/4 (+ 1: the blocks then start in different
    // bank halves) rows of 16 p; and exp(+2 pi i k / N)
    constexpr int kZRows = 8 * ZG + 1;
    __shared__ float2 zbuf[ZINV ? kWaves * 2 * kZRows * 16 : 1];
    __shared__ float2 ztw[ZINV ? 32 * ZG : 1];

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, n = lane & 15;
    const int Q = T.N >> 2;
    const long vol = (long)T.N * T.P;
    const int nred = BWD ? T.fo : T.f, nout = BWD ? T.f : T.fo;

    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int q_ = (slot / T.ngroups) * 8 + xcd, og = slot % T.ngroups;
    if (q_ >= T.nq) return;
    const int ptiles = (T.P + 15) >> 4;
    const int pt = q_ % ptiles, sb = q_ / ptiles;
    const int p0 = pt * 16;
    const bool pvalid = p0 + n < T.P;
    const int zgrp0 = sb * ZG;                          // first z0-group of this workgroup's slice
    const int o0 = (og * kWaves + wave) * G;            // the waves differ in their result nodes

    // ---- A operands: twiddles of (z0-group t, class c, k-step s); lane holds A[m = lane % 16][k = lane / 16]
    float A[ZG][NB > 0 ? NB : 1];
    {
        const int m = lane & 15, kk0 = lane >> 4;
#pragma unroll
        for (int t = 0; t < ZG; ++t) {
            const int z0 = (zgrp0 + t) * 8 + (m >> 1);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
#pragma unroll
                for (int s = 0; s < class_steps(KZ, c); ++s) {
                    const int kk = 4 * s + kk0;
                    const int a = c + 4 * (kk >> 1);
                    float v = 0.f;
                    if (a < KZ) {
                        const int idx = (a * z0) % T.N;
                        float sn, cs;
                        sincospif(2.0f * (float)idx / (float)T.N, &sn, &cs);
                        // V = w exp(-i th): re = w.re cos + w.im sin, im = w.im cos - w.re sin
                        v = (m & 1) == (kk & 1) ? cs : ((m & 1) ? -sn : sn);
                    }
                    A[t][steps_before(KZ, c) + s] = v;
                }
            }
        }
    }

    // ---- B operands: lane (g, n) supplies row k = g of every k-step: tap a = c + 8 s + 4 (g / 2), component g % 2
    // Rows past the last tap meet a zero in A and lanes past the last p own a column nobody stores, so
    // both simply load a finite value from a clamped address: no branch around any load.
    int boff[NB > 0 ? NB : 1];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int s = 0; s < class_steps(KZ, c); ++s) {
            const int a = min(c + 8 * s + 4 * (g >> 1), KZ - 1);
            boff[steps_before(KZ, c) + s] = (a * T.P + min(p0 + n, T.P - 1)) * 2 + (g & 1);
        }
    const float* whf = reinterpret_cast<const float*>(T.Wh);
    const long wplane = (long)KZ * T.P * 2;             // floats per pair

    // ---- node-spectrum tile: the rows z = 8 (first z0-group of the workgroup) + 0 .. 8 ZG - 1, + q N/4 for
    // q = 0..3, x 16 p.  A read takes, for one e, the rows 2 g + e of an 8-row block for the four lane groups g:
    // so within a block the rows are stored in the order 0, 2, 4, 6, 1, 3, 5, 7 (row 2 g + e at place 4 e + g) and
    // a read covers 512 consecutive bytes, free of bank conflicts (in natural order the four rows are 256 bytes
    // apart and share their banks).  float2 index: ((q * ZG + block) * 8 + place) * 16 + p.
    // The tile travels global -> LDS directly (no registers): 16 bytes per lane and load where rows start on
    // 16-byte boundaries (P even: a wave-load fills a block), else 4 bytes (two places); which spectrum element
    // a lane fetches splits into a per-lane part, worked out once, and a part that depends on the load only
    // (scalar).  Lanes beyond the last in-plane frequency never load; their words keep the zeros written here.
    constexpr int kRowsQ = 8 * ZG;                      // rows per quarter-period block
    const int tile = 4 * kRowsQ * 16;                   // float2 per buffer
    for (int i = threadIdx.x; i < tile; i += 64 * kWaves) tileA[i] = tileB[i] = make_float2(0.f, 0.f);
    if (T.N < 0) tileA[threadIdx.x] = tileB[threadIdx.x] = T.X[threadIdx.x];    // never taken: tells the optimizer that LDS holds data
    if (ZINV && (int)threadIdx.x < 32 * ZG) {
        float sn, cs;
        sincospif(2.0f * (float)threadIdx.x / (float)(32 * ZG), &sn, &cs);
        ztw[threadIdx.x] = make_float2(cs, sn);
    }
    const float* xf = reinterpret_cast<const float*>(T.X);
    const bool wide = (T.P & 1) == 0;                   // uniform
    const int zbase = sb * kRowsQ;                      // first row of the workgroup's slice (one slice per workgroup)
    unsigned xthread;                                   // byte offset of this lane's element of load 0 inside a node spectrum
    bool xvalid;
    if (wide) {
        // lane -> place lane / 8 of the block, 16-byte segment lane % 8 of the row
        const int place = lane >> 3, pp = p0 + 2 * (lane & 7);
        xvalid = pp < T.P;
        xthread = (unsigned)(((long)(zbase + 2 * (place & 3) + (place >> 2)) * T.P + pp) * 8);
    } else {
        // lane -> place 2 (k % 4) + lane / 32 of the block (k: the load), float lane % 32 of the row
        const int pp = p0 + ((lane & 31) >> 1);
        xvalid = pp < T.P;
        xthread = (unsigned)(((long)(zbase + 2 * (lane >> 5)) * T.P + pp) * 8 + (lane & 1) * 4);
    }
    auto fetch_tile = [&](int r, float2* buf) {
        const char* xb = reinterpret_cast<const char*>(xf + (long)r * vol * 2);     // uniform
        float* dst = reinterpret_cast<float*>(buf);
        // (the empty asm makes the lane's offset a value of this reduction index: otherwise the optimizer forms
        // every load's 64-bit address once, outside the reduction loop, and keeps them all in registers, which
        // costs the small kernels a wave of occupancy)
        unsigned xt = xthread;
        asm volatile("" : "+v"(xt));
        if (wide) {
#pragma unroll
            for (int j = 0; j < ZG; ++j) {
                const int k = wave + kWaves * j;                                    // uniform: block k % ZG of quarter k / ZG
                const unsigned ck = (unsigned)(((long)(8 * (k % ZG) + (k / ZG) * Q) * T.P) * 8);
                if (xvalid)
                    __builtin_amdgcn_global_load_lds((global_cptr)(xb + (ck + xt)), (lds_ptr)(dst + k * 256), 16, 0, 0);
            }
        } else {
            auto load_rows = [&](int j) {
                const int k = wave + kWaves * j;                                    // uniform: places 2 (k % 4), + 1 of block k / 4
                const int blk = k >> 2, kk = k & 3;
                // place 2 kk + h holds row 2 ((2 kk + h) % 4) + (2 kk + h) / 4 = 4 (kk % 2) + 2 h + kk / 2
                const unsigned ck = (unsigned)(((long)(8 * (blk % ZG) + (blk / ZG) * Q + 4 * (kk & 1) + (kk >> 1)) * T.P) * 8);
                if (xvalid)
                    __builtin_amdgcn_global_load_lds((global_cptr)(xb + (ck + xt)), (lds_ptr)(dst + k * 64), 4, 0, 0);
            };
            // four loads per wave unrolled, more of them rolled (unrolled they cost registers: a wave of occupancy
            // for the kernels that have three)
            if constexpr (ZG == 1) {
#pragma unroll
                for (int j = 0; j < 4; ++j) load_rows(j);
            } else {
#pragma nounroll
                for (int j = 0; j < 4 * ZG; ++j) load_rows(j);
            }
        }
    };

    float2 acc[G][ZG][2][4];
#pragma unroll
    for (int gi = 0; gi < G; ++gi)
#pragma unroll
        for (int t = 0; t < ZG; ++t)
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[gi][t][e][q] = make_float2(0.f, 0.f);

    // pair of (reduction index r, result node o); kernels are stored [f'][f]
    auto pair_base = [&](int r, int gi) {
        const int o = min(o0 + gi, nout - 1);
        const long pair = BWD ? (long)r * T.f + o : (long)o * T.f + r;
        return whf + pair * wplane;
    };
    float b0[G][NB > 0 ? NB : 1], b1[G][NB > 0 ? NB : 1];      // two operand sets taking turns
    auto load_b = [&](int r, float (&b)[G][NB > 0 ? NB : 1]) {
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
            const float* wb = pair_base(r, gi);
#pragma unroll
            for (int k = 0; k < NB; ++k) b[gi][k] = wb[boff[k]];
        }
    };

    __syncthreads();                    // the zeros are in place
    fetch_tile(0, tileA);
    load_b(0, b0);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    int xo = g * 16 + n;                                            // this lane's element of place g (row 2 g) of a block

    // one reduction index: reads the tile in `cur` while the next one lands in `nxt`
    auto reduction_step = [&](int r, const float2* cur, float2* nxt, float (&bcur)[G][NB > 0 ? NB : 1],
                              float (&bnext)[G][NB > 0 ? NB : 1]) {
        if (r + 1 < nred) {
            fetch_tile(r + 1, nxt);
            load_b(r + 1, bnext);
        }
        // The ZG * G (z0-group, result node) groups of this reduction index, in order, software
        // pipelined by one: the matrix products of group k + 1 are issued before the vector work of
        // group k, so their latency is covered.  Left alone the compiler starts the products of all
        // groups at once and runs out of registers; the empty asm at the end of a group takes the
        // group's sums and an operand of the group after the next as in-out operands, so nothing
        // beyond the next group can be moved above it.
        constexpr int K = ZG * G;
        auto class_sums = [&](int k, floatx4 (&D)[4]) {
            const int t = k / G, gi = k % G;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                D[c] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < class_steps(KZ, c); ++s)
                    D[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(A[t][steps_before(KZ, c) + s],
                                                                bcur[gi][steps_before(KZ, c) + s], D[c], 0, 0, 0);
            }
        };
        auto load_x = [&](int t, float2 (&x)[2][4]) {
            const float2* myx = cur + xo;
#pragma unroll
            for (int e = 0; e < 2; ++e)
#pragma unroll
                for (int q = 0; q < 4; ++q) x[e][q] = myx[(q * kRowsQ + 8 * t + 4 * e) * 16];
        };
        floatx4 D0[4], D1[4];
        float2 x0[2][4], x1[2][4];
        load_x(0, x0);
        class_sums(0, D0);
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const int t = k / G, gi = k % G;
            floatx4 (&D)[4] = (k & 1) ? D1 : D0;
            floatx4 (&Dn)[4] = (k & 1) ? D0 : D1;
            float2 (&x)[2][4] = (t & 1) ? x1 : x0;
            if (k + 1 < K) {
                if ((k + 1) % G == 0) load_x(t + 1, (t & 1) ? x0 : x1);
                class_sums(k + 1, Dn);
            }
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                // radix-4 butterfly: W^_q = sum_c V_c (-i)^(c q)
                const float2 v0 = make_float2(D[0][2 * e], D[0][2 * e + 1]);
                const float2 v1 = make_float2(D[1][2 * e], D[1][2 * e + 1]);
                const float2 v2 = make_float2(D[2][2 * e], D[2][2 * e + 1]);
                const float2 v3 = make_float2(D[3][2 * e], D[3][2 * e + 1]);
                const float2 s02 = make_float2(v0.x + v2.x, v0.y + v2.y);
                const float2 d02 = make_float2(v0.x - v2.x, v0.y - v2.y);
                const float2 s13 = make_float2(v1.x + v3.x, v1.y + v3.y);
                const float2 d13 = make_float2(v1.x - v3.x, v1.y - v3.y);
                float2 wq[4];
                wq[0] = make_float2(s02.x + s13.x, s02.y + s13.y);
                wq[2] = make_float2(s02.x - s13.x, s02.y - s13.y);
                wq[1] = make_float2(d02.x + d13.y, d02.y - d13.x);      // d02 - i d13
                wq[3] = make_float2(d02.x - d13.y, d02.y + d13.x);      // d02 + i d13
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float2 xv = x[e][q];
                    float2& a = acc[gi][t][e][q];
                    if (BWD) {      // conj(W^) x
                        a.x = fmaf(wq[q].x, xv.x, fmaf(wq[q].y, xv.y, a.x));
                        a.y = fmaf(wq[q].x, xv.y, fmaf(-wq[q].y, xv.x, a.y));
                    } else {
                        a.x = fmaf(wq[q].x, xv.x, fmaf(-wq[q].y, xv.y, a.x));
                        a.y = fmaf(wq[q].x, xv.y, fmaf(wq[q].y, xv.x, a.y));
                    }
                }
            }
            float2 (&ag)[2][4] = acc[gi][t];
            asm volatile("" : "+v"(ag[0][0].x), "+v"(ag[0][0].y), "+v"(ag[0][1].x), "+v"(ag[0][1].y),
                              "+v"(ag[0][2].x), "+v"(ag[0][2].y), "+v"(ag[0][3].x), "+v"(ag[0][3].y),
                              "+v"(ag[1][0].x), "+v"(ag[1][0].y), "+v"(ag[1][1].x), "+v"(ag[1][1].y),
                              "+v"(ag[1][2].x), "+v"(ag[1][2].y), "+v"(ag[1][3].x), "+v"(ag[1][3].y),
                              "+v"(xo), "+v"(bcur[(k + 2) % G][0]));
        }
        __builtin_amdgcn_s_waitcnt(0);      // this wave's part of the next tile has landed
        __syncthreads();                    // everyone's has, and nobody still reads the current one
    };
    // two steps per trip, so that each copy of the code names its buffers statically
    for (int r = 0; r < nred; r += 2) {
        reduction_step(r, tileA, tileB, b0, b1);
        if (r + 1 < nred) reduction_step(r + 1, tileB, tileA, b1, b0);
    }

    if constexpr (ZINV) {
        constexpr int Q4 = 8 * ZG;
        float2* zb = zbuf + wave * (2 * kZRows * 16);
        const int h = (lane >> 4) & 1;
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
            if (o0 + gi >= nout) break;
            float2* yb = T.Y + (long)(o0 + gi) * vol + p0 + n;
#pragma unroll
            for (int mp = 0; mp < 2; ++mp) {
                // U[z0][m0] = exp(+2 pi i z0 m0 / N) sum_q Y[q N/4 + z0] i^(q m0) for m0 = 2 mp and 2 mp + 1 and
                // this lane's z0 = 8 t + 2 g + e into the wave's piece of LDS (row z0 at place 8 t + 4 e + g: the
                // lane groups g then write consecutive rows); then lane (h, n), h < 2, takes the N/4 values of
                // m0 = 2 mp + h at its p.  The LDS operations of a wave complete in the order of issue, so a
                // round's reads see its writes and the next round's writes come after its reads.
#pragma unroll
                for (int t = 0; t < ZG; ++t)
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const float2 (&y)[4] = acc[gi][t][e];
                        const int z0 = 8 * t + 2 * g + e;
                        float2 u0, u1;
                        if (mp == 0) {
                            u0 = cadd(cadd(y[0], y[2]), cadd(y[1], y[3]));
                            const float2 d02 = csub(y[0], y[2]), d13 = csub(y[1], y[3]);
                            u1 = make_float2(d02.x - d13.y, d02.y + d13.x);     // d02 + i d13
                        } else {
                            u0 = csub(cadd(y[0], y[2]), cadd(y[1], y[3]));
                            const float2 d02 = csub(y[0], y[2]), d13 = csub(y[1], y[3]);
                            u1 = make_float2(d02.x + d13.y, d02.y - d13.x);     // d02 - i d13
                            const float2 w = ztw[2 * z0];
                            u0 = make_float2(u0.x * w.x - u0.y * w.y, u0.x * w.y + u0.y * w.x);
                        }
                        const float2 w = ztw[(2 * mp + 1) * z0];                // z0 m0 < 3 N / 4
                        u1 = make_float2(u1.x * w.x - u1.y * w.y, u1.x * w.y + u1.y * w.x);
                        zb[(8 * t + 4 * e + g) * 16 + n] = u0;
                        zb[(kZRows + 8 * t + 4 * e + g) * 16 + n] = u1;
                    }
                if (lane < 32) {
                    float2 x[Q4], y[Q4];
#pragma unroll
                    for (int z0 = 0; z0 < Q4; ++z0)
                        x[z0] = zb[(h * kZRows + 8 * (z0 >> 3) + 4 * (z0 & 1) + ((z0 >> 1) & 3)) * 16 + n];
                    passes<Q4, +1, Q4, 1>(x, y);
                    constexpr bool in_y = (count_passes(Q4) % 2) == 1;
                    if (pvalid) {
#pragma unroll
                        for (int m1 = 0; m1 < Q4; ++m1) {
                            const int z = 2 * mp + h + 4 * m1;
                            if (z >= T.zinv_o0 && z < T.zinv_o0 + T.zinv_no) yb[(long)z * T.P] = in_y ? y[m1] : x[m1];
                        }
                    }
                }
            }
        }
    } else {
        if (!pvalid) return;
#pragma unroll
        for (int gi = 0; gi < G; ++gi) {
            if (o0 + gi >= nout) break;
            float2* yb = T.Y + (long)(o0 + gi) * vol + p0 + n;
#pragma unroll
            for (int t = 0; t < ZG; ++t)
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int z0 = (zgrp0 + t) * 8 + 2 * g + e;
#pragma unroll
                    for (int q = 0; q < 4; ++q) yb[(long)(z0 + q * Q) * T.P] = acc[gi][t][e][q];
                }
        }
    }
}

template <bool BWD, int KZ, int ZG, bool ZINV>
int launch_zg(MacTile T, int nout, hipStream_t s)
{
    T.ngroups = (nout + kWaves * kG - 1) / (kWaves * kG);
    const long blocks = ((long)(T.nq + 7) / 8) * 8 * T.ngroups;
    if (blocks >= 2147483647L) return fail(ZNN_EUNSUPPORTED, "too many frequencies");
    ZNN_LAUNCH(BWD ? "spectral mac backward (taps folded in, MFMA)" : "spectral mac forward (taps folded in, MFMA)", s,
               (k_mac_mfma<BWD, KZ, ZG, ZINV>), dim3((unsigned)blocks), dim3(64 * kWaves), 0, T);
    return check_launch("spectral multiply-accumulate");
}

template <bool BWD, int KZ>
int launch_kz(MacTile T, int ZG, int nout, hipStream_t s)
{
    if (T.zinv_no > 0) {
        if (ZG == 3) return launch_zg<BWD, KZ, 3, true>(T, nout, s);
        if (ZG == 2) return launch_zg<BWD, KZ, 2, true>(T, nout, s);
        return launch_zg<BWD, KZ, 1, true>(T, nout, s);
    }
    if (ZG == 3) return launch_zg<BWD, KZ, 3, false>(T, nout, s);
    if (ZG == 2) return launch_zg<BWD, KZ, 2, false>(T, nout, s);
    return launch_zg<BWD, KZ, 1, false>(T, nout, s);
}

template <bool BWD>
int launch_dir(int taps, MacTile T, int ZG, int nout, hipStream_t s)
{
    switch (taps) {
        case 1: return launch_kz<BWD, 1>(T, ZG, nout, s);
        case 2: return launch_kz<BWD, 2>(T, ZG, nout, s);
        case 3: return launch_kz<BWD, 3>(T, ZG, nout, s);
        case 4: return launch_kz<BWD, 4>(T, ZG, nout, s);
        case 5: return launch_kz<BWD, 5>(T, ZG, nout, s);
        case 6: return launch_kz<BWD, 6>(T, ZG, nout, s);
        case 7: return launch_kz<BWD, 7>(T, ZG, nout, s);
        case 8: return launch_kz<BWD, 8>(T, ZG, nout, s);
        case 9: return launch_kz<BWD, 9>(T, ZG, nout, s);
        case 10: return launch_kz<BWD, 10>(T, ZG, nout, s);
        case 11: return launch_kz<BWD, 11>(T, ZG, nout, s);
        case 12: return launch_kz<BWD, 12>(T, ZG, nout, s);
        case 13: return launch_kz<BWD, 13>(T, ZG, nout, s);
        case 14: return launch_kz<BWD, 14>(T, ZG, nout, s);
        case 15: return launch_kz<BWD, 15>(T, ZG, nout, s);
        case 16: return launch_kz<BWD, 16>(T, ZG, nout, s);
        default: return fail(ZNN_EUNSUPPORTED, "more taps than the folded multiply-accumulate takes");
    }
}

}  // namespace

bool fft_mac_mfma_supported(int taps, int N, int P)
{
    // offsets inside one node spectrum (N * P elements) and inside one pair's half spectrum
    // (taps * P elements) are 32-bit
    return N % 32 == 0 && taps >= 1 && taps <= kMaxFoldedTaps && (long)taps * P * 2 < 2147483647L &&
           (long)N * P * 8 < 4294967296L;       // a thread's byte offset inside a node spectrum fits 32 bits
}

namespace {

// z0-groups per wave
int groups_per_wave(int N, int P, int nout)
{
    // z0-groups per wave: as many as divide the axis (every half-spectrum element is then loaded by fewer
    // waves) while the launch still has two waves per SIMD; small layers take fewer groups per wave instead
    // (the 2D benchmark layer: 1440 -> 2880 waves, 0.213 -> 0.165 ms).  One slice per workgroup: its four waves
    // then share one node-spectrum tile for eight result nodes (two slices and four nodes measured 8 % slower).
    const int groups = N / 32;
    const long per_slice = (long)((P + 15) / 16) * ((nout + 1) / 2);
    for (int z = 3; z >= 2; --z)
        if (groups % z == 0 && per_slice * (groups / z) >= 2048) return z;
    return 1;
}

}  // namespace

bool fft_mac_mfma_can_invert(int taps, int N, int P, int nout)
{
    return fft_mac_mfma_supported(taps, N, P) && 32 * groups_per_wave(N, P, nout) == N;
}

int fft_mac_mfma(bool backward, int taps, int f, int fo, int N, int P, const float2* Wh, const float2* X,
                 float2* Y, int zinv_o0, int zinv_no, hipStream_t s)
{
    if (!fft_mac_mfma_supported(taps, N, P)) return fail(ZNN_EUNSUPPORTED, "layer does not fit the MFMA multiply-accumulate");
    MacTile T = {};
    T.Wh = Wh; T.X = X; T.Y = Y;
    T.f = f; T.fo = fo; T.N = N; T.P = P;
    const int groups = N / 32;
    const int nout = backward ? f : fo;
    const int ZG = groups_per_wave(N, P, nout);
    if (zinv_no > 0 && 32 * ZG != N) return fail(ZNN_EINVAL, "a wave does not own the whole folded axis: no inverse transform in the multiply-accumulate");
    T.zinv_o0 = zinv_o0; T.zinv_no = zinv_no > 0 ? zinv_no : 0;
    T.nslice = groups / ZG;
    T.nq = ((P + 15) / 16) * T.nslice;
    return backward ? launch_dir<true>(taps, T, ZG, nout, s) : launch_dir<false>(taps, T, ZG, nout, s);
}

}  // namespace znn
