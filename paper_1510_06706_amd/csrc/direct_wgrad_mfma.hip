// Direct method, kernel gradient (Section 3.2) on the fp32 matrix cores.
//
//   gw[j][i][a][b][c] = sum_v gout[j][v] * in[i][v + (kz-1-a, ky-1-b, kx-1-c)]
//
// is a GEMM whose reduction runs over the output voxels v:
//
//   D[m][n] += A[m][k] * B[k][n]      v_mfma_f32_16x16x4_f32
//     m : 16 output maps j                    (A = gout, from an LDS tile)
//     n : 16 columns of the flattened (c, i)  (B = in shifted by the tap, from an LDS tile)
//     k : 4 consecutive output voxels of one x-row
//
// A workgroup owns one (a, b) tap plane, a group of columns n = c*f + i and a
// share of the voxel rows (split-K).  Tiles of R voxel rows travel from global
// memory straight into LDS (global_load_lds, no registers in between) into one
// of two buffers, so the next tile is in flight while the four waves run the
// MFMAs of the current one.  The waves take alternate 4-voxel steps of a tile;
// their accumulators are added in a fixed order through LDS and written as one
// partial matrix per workgroup.  A second kernel adds the partial matrices in
// ascending split order, so the result is bit-reproducible (no atomics).
#include <cstdio>
#include <cstdlib>
#include <type_traits>

#include "znn_internal.h"

namespace znn {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) const void* global_cptr;
typedef __attribute__((address_space(3))) void* lds_ptr;

// Two tile buffers as separate LDS objects: the compiler then knows that loads
// landing in one buffer do not alias reads of the other and lets them overlap.
constexpr int kBufFloats = 18432;                 // 72 KiB each

struct WgradTile {
    const float* in; const float* gout; float* partial;
    int f, fo;
    int nz, ny, nx;
    int oz, oy, ox;
    int kz, ky, kx;
    int spz, spy, spx;  // sparsity: taps are this many voxels apart
    int TX, XT, R;      // x-segment width (multiple of 4), segments per row, rows per tile
    int GS, IS, TXH;    // LDS strides: gout map, in map, in row
    int Mpad, Npad;     // padded partial-matrix extents
    int G;              // column groups
    int tiles, tps;     // voxel tiles in total and per split
    int AB;             // kz * ky
    FastDiv dTX, dTXH, dOY;
    int vec4;           // 16-byte global->LDS loads are legal for this shape
    int fast;           // the tile loader may use offsets worked out once per workgroup (see the kernel)
    int mapmajor;       // GEMM columns ordered n = i*kx + c instead of n = c*f + i (see choose_wgrad)
    FastDiv dGS, dIS;
};

// The MFMAs of this wave's share of one staged tile.  A step covers 8 consecutive voxels:
// lane group g (= lane/16) reads the voxel pair (2g, 2g+1) of every operand with one
// two-dword LDS read and feeds two MFMAs from it.  The wave takes steps kp, kp+4, ... < k1.
// Two register sets take turns, so the LDS reads of the next step are queued before the
// MFMAs of the current one and only waited for after them; the code is kept free of
// branches around loads and MFMAs (a step past the end re-reads the last one, NTA is the
// compile-time number of column tiles that hold real columns) because the compiler can
// only count outstanding loads exactly in straight-line code.  NTA < 0: the number of
// live tiles is the run-time value ntw (any ragged column group; slower).
template <int NJ, int NT, int NTA>
__device__ __forceinline__ void wgrad_steps(floatx4 (&acc)[NJ][NT], const float* buf, const int (&aoff)[NJ],
                                            const int (&boff)[NT], int kp, int k1, int grp, FastDiv dTX, int TX,
                                            int TXH, int ntw)
{
    if (kp >= k1) return;
    const int klast = kp + ((k1 - 1 - kp) & ~3);
    auto load_step = [&](int k, float2 (&av)[NJ], float2 (&bv)[NT]) {
        const int e = 8 * k + 2 * grp;
        const int r = (int)fdiv((unsigned)e, dTX), x = e - r * TX;
        const int ao = e, bo = r * TXH + x;
#pragma unroll
        for (int jt = 0; jt < NJ; ++jt) av[jt] = make_float2(buf[aoff[jt] + ao], buf[aoff[jt] + ao + 1]);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            if (NTA < 0 || nt < NTA) bv[nt] = make_float2(buf[boff[nt] + bo], buf[boff[nt] + bo + 1]);
    };
    // first voxel of every pair for all tiles, then the second: consecutive MFMAs never wait
    // for each other's accumulator
    auto mfma_step = [&](const float2 (&av)[NJ], const float2 (&bv)[NT]) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            if (NTA < 0 ? nt < ntw : nt < NTA) {
#pragma unroll
                for (int jt = 0; jt < NJ; ++jt)
                    acc[jt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[jt].x, bv[nt].x, acc[jt][nt], 0, 0, 0);
            }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            if (NTA < 0 ? nt < ntw : nt < NTA) {
#pragma unroll
                for (int jt = 0; jt < NJ; ++jt)
                    acc[jt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[jt].y, bv[nt].y, acc[jt][nt], 0, 0, 0);
            }
    };
    float2 a0[NJ], b0[NT], a1[NJ], b1[NT];
    load_step(kp, a0, b0);
    for (;;) {
        load_step(min(kp + 4, klast), a1, b1);
        mfma_step(a0, b0);
        if (kp + 4 >= k1) break;
        load_step(min(kp + 8, klast), a0, b0);
        mfma_step(a1, b1);
        if (kp + 8 >= k1) break;
        kp += 8;
    }
}

// NH = 1: four waves share every column tile and split the voxel steps four ways.
// NH = 2: eight waves; waves 0-3 own the first NT column tiles of the group, waves 4-7 the
// next NT, and each half splits the voxel steps four ways.  Two waves per SIMD: while one
// waits for its global->LDS loads to be queued the other keeps the matrix cores busy.
template <int NJ, int NT, int NH>
__global__ void __launch_bounds__(256 * NH) k_wgrad_mfma(WgradTile P)
{
    constexpr int NW = 4 * NH;
    __shared__ __attribute__((aligned(16))) float bufA[kBufFloats];
    __shared__ __attribute__((aligned(16))) float bufB[kBufFloats];
    // The tile buffers are filled by global_load_lds only, which the optimizer does not
    // count as a store to them; this never-taken ordinary store keeps their contents
    // "unknown" instead of "never written".
    if (P.tiles < 0) {
        bufA[threadIdx.x] = P.in[threadIdx.x];
        bufB[threadIdx.x] = P.gout[threadIdx.x];
    }
    // the wave index is the same in all 64 lanes: telling the compiler so keeps everything
    // derived from it (loop counters, tile predicates) in scalar registers and branches
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int half = wave >> 2, kw = wave & 3;
    const int col = lane & 15, grp = lane >> 4;
    const int s = blockIdx.x, ab = blockIdx.y;
    const int a = ab / P.ky, b = ab % P.ky;
    const int cg = blockIdx.z % P.G, jg = blockIdx.z / P.G;
    const int ncols = P.f * P.kx;
    const int n0 = cg * NT * NH * 16;
    const int n1 = min(n0 + NT * NH * 16, ncols);
    // the group's range of x-taps [cmin, cmax] and of input maps [imin, imax]
    int cmin, cmax, imin, imax;
    if (P.mapmajor) {
        imin = n0 / P.kx; imax = (n1 - 1) / P.kx;
        cmin = 0; cmax = P.kx - 1;
        if (imin == imax) { cmin = n0 % P.kx; cmax = (n1 - 1) % P.kx; }
    } else {
        cmin = n0 / P.f; cmax = (n1 - 1) / P.f;
        imin = 0; imax = P.f - 1;
        if (cmin == cmax) { imin = n0 % P.f; imax = (n1 - 1) % P.f; }
    }
    const int nmaps = imax - imin + 1;
    const int TXH = P.TXH;
    const int itoff = NJ * 16 * P.GS;       // the in tile follows the gout tile in a buffer

    int aoff[NJ], boff[NT];
#pragma unroll
    for (int jt = 0; jt < NJ; ++jt) aoff[jt] = (jt * 16 + col) * P.GS;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int n = n0 + (half * NT + nt) * 16 + col;
        int o = 0;
        if (n < n1) {
            const int c = P.mapmajor ? n % P.kx : n / P.f, i = P.mapmajor ? n / P.kx : n % P.f;
            o = (i - imin) * P.IS + (cmax - c) * P.spx;
        }
        boff[nt] = itoff + o;
    }

    // column tiles of this half that hold real columns (wave-uniform): the rest is skipped
    const int ntw = max(0, min(NT, ((n1 - n0 + 15) >> 4) - half * NT));

    floatx4 acc[NJ][NT];
#pragma unroll
    for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[jt][nt] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int rows = P.oz * P.oy;
    const long oplane = (long)rows * P.ox;
    const long iplane = (long)P.ny * P.nx;
    const long ivol = (long)P.nz * iplane;
    const int t_end = min((s + 1) * P.tps, P.tiles);
    const int RT = P.R * P.TX, RTH = P.R * TXH;
    // 8-voxel steps per tile.  R * TX is a multiple of 4; when it is no multiple of 8 the last step
    // runs half into the padding behind a map row, which holds zeros in the gout tile.
    const int nkp = (RT + 7) / 8;
    // Both buffers are zeroed once: the loaders never write padding (rows of maps past the last real
    // one, words behind a row's voxels, lanes outside the images on tiles that have none), so it
    // stays zero, and whatever an MFMA step reads next to a zero gout word is a finite number.
    const int mreal = min(NJ * 16, P.fo - jg * NJ * 16);
    for (int q = threadIdx.x; q < kBufFloats; q += 64 * NW) { bufA[q] = 0.f; bufB[q] = 0.f; }
    __syncthreads();

    // Queue the global->LDS loads of one tile.  A wave-load moves 64 * W consecutive tile
    // elements of one map (W = 4: 16-byte loads, legal when every group of four x-neighbours
    // is entirely inside or outside the image, P.vec4).  The vector arithmetic is kept to one
    // byte offset per lane and 64 * W elements, shared by all maps: the map bases are wave-
    // uniform (scalar registers), lanes outside the images are masked off the load, and only
    // tiles that have such lanes store zeros for them.  (Vector instructions issued here hold
    // up the other waves' MFMAs on the same SIMD.)
    auto issue_part = [&](float* dst, int stride, const float* base, long mapvol, int nm, int width, int total,
                          FastDiv dw, int rho0, int xg0, int xlim, bool is_in, auto WT) {
        constexpr int W = decltype(WT)::value;
        for (int k = 0; k * 64 * W < total; ++k) {
            const int e = k * 64 * W + lane * W;
            const int r = (int)fdiv((unsigned)e, dw), x = e - r * width;
            const int rho = rho0 + r, gx = xg0 + x;
            const bool inside = e < total;
            const bool ok = inside && rho < rows && gx < xlim;
            unsigned voff;
            if (is_in) {
                const int z = (int)fdiv((unsigned)rho, P.dOY), y = rho - z * P.oy;
                voff = (unsigned)((z + (P.kz - 1 - a) * P.spz) * (int)iplane + (y + (P.ky - 1 - b) * P.spy) * P.nx + gx) * 4u;
            } else {
                voff = (unsigned)(rho * P.ox + gx) * 4u;
            }
            const bool fix = inside && !ok;
            const bool anyfix = __builtin_amdgcn_ballot_w64(fix) != 0;      // wave-uniform
            for (int m = wave; m < nm; m += NW) {
                const char* mb = reinterpret_cast<const char*>(base + (long)m * mapvol);   // uniform
                float* row = dst + m * stride + k * 64 * W;                                 // uniform
                if (ok) {
                    if constexpr (W == 4) __builtin_amdgcn_global_load_lds((global_cptr)(mb + voff), (lds_ptr)row, 16, 0, 0);
                    else __builtin_amdgcn_global_load_lds((global_cptr)(mb + voff), (lds_ptr)row, 4, 0, 0);
                }
                if (anyfix && fix) {
#pragma unroll
                    for (int q = 0; q < W; ++q) row[lane * W + q] = 0.f;
                }
            }
        }
    };
    // Fast loader (P.fast, decided on the host: one x-segment per row, 16-byte loads, tiles that
    // neither straddle a z-plane nor end behind the last row).  A wave-load then fills 256
    // consecutive floats of a tile region regardless of where map rows begin and end; which map and
    // which voxel a lane's four floats belong to is the same for every tile, so the lane's byte offset
    // from the tile's origin and its validity are worked out once, here, and a tile costs this wave a
    // handful of loads with no vector arithmetic at all.  Spans are dealt to the waves round-robin.
    constexpr int kMaxSpans = 5;
    unsigned fg_off[kMaxSpans], fi_off[kMaxSpans];
    bool fg_ok[kMaxSpans], fi_ok[kMaxSpans];
    const int nspan_g = (mreal * P.GS + 255) >> 8, nspan_i = (nmaps * P.IS + 255) >> 8;
    if (P.fast) {
#pragma unroll
        for (int q = 0; q < kMaxSpans; ++q) {
            const int L = (wave + q * NW) * 256 + lane * 4;
            {
                const int m = (int)fdiv((unsigned)L, P.dGS), e = L - m * P.GS;
                const int r = (int)fdiv((unsigned)e, P.dTX), x = e - r * P.TX;
                fg_ok[q] = m < mreal && e < RT && x < P.ox;
                fg_off[q] = (unsigned)(m * (int)oplane + r * P.ox + x) * 4u;
            }
            {
                const int m = (int)fdiv((unsigned)L, P.dIS), e = L - m * P.IS;
                const int r = (int)fdiv((unsigned)e, P.dTXH), x = e - r * TXH;
                const int ix = (P.kx - 1 - cmax) * P.spx + x;
                fi_ok[q] = m < nmaps && e < RTH && ix < P.nx;
                fi_off[q] = (unsigned)(m * (int)ivol + r * P.nx + ix) * 4u;
            }
        }
    }
    auto issue_tile_fast = [&](int tile, float* buf) {
        const int rho0 = tile * P.R;                                    // XT == 1
        const int z = (int)fdiv((unsigned)rho0, P.dOY), y = rho0 - z * P.oy;
        const char* gb = reinterpret_cast<const char*>(P.gout + (long)(jg * NJ * 16) * oplane + (long)rho0 * P.ox);
        const char* ib = reinterpret_cast<const char*>(P.in + (long)imin * ivol + (long)(z + (P.kz - 1 - a) * P.spz) * iplane +
                                                       (long)(y + (P.ky - 1 - b) * P.spy) * P.nx);
#pragma unroll
        for (int q = 0; q < kMaxSpans; ++q) {
            const int sp = wave + q * NW;                               // uniform
            if (sp < nspan_g && fg_ok[q])
                __builtin_amdgcn_global_load_lds((global_cptr)(gb + fg_off[q]), (lds_ptr)(buf + sp * 256), 16, 0, 0);
        }
#pragma unroll
        for (int q = 0; q < kMaxSpans; ++q) {
            const int sp = wave + q * NW;
            if (sp < nspan_i && fi_ok[q])
                __builtin_amdgcn_global_load_lds((global_cptr)(ib + fi_off[q]), (lds_ptr)(buf + itoff + sp * 256), 16, 0, 0);
        }
    };
    auto issue_tile = [&](int tile, float* buf) {
        if (P.fast) { issue_tile_fast(tile, buf); return; }
        const int xt = tile % P.XT, rt = tile / P.XT;
        const int rho0 = rt * P.R, xs0 = xt * P.TX;
        const int xin0 = xs0 + (P.kx - 1 - cmax) * P.spx;
        const float* gbase = P.gout + (long)(jg * NJ * 16) * oplane;
        const float* ibase = P.in + (long)imin * ivol;
        if (P.vec4) {
            issue_part(buf, P.GS, gbase, oplane, mreal, P.TX, RT, P.dTX, rho0, xs0, P.ox, false, std::integral_constant<int, 4>{});
            issue_part(buf + itoff, P.IS, ibase, ivol, nmaps, TXH, RTH, P.dTXH, rho0, xin0, P.nx, true, std::integral_constant<int, 4>{});
        } else {
            issue_part(buf, P.GS, gbase, oplane, mreal, P.TX, RT, P.dTX, rho0, xs0, P.ox, false, std::integral_constant<int, 1>{});
            issue_part(buf + itoff, P.IS, ibase, ivol, nmaps, TXH, RTH, P.dTXH, rho0, xin0, P.nx, true, std::integral_constant<int, 1>{});
        }
    };

    // The whole tile loop is instantiated once per variant of the MFMA steps (all column tiles
    // live, one padded tile skipped, run-time count) and the variant is chosen once, out here:
    // choosing per tile would merge the variants' register assignments after every tile, which
    // costs a copy of every accumulator (vector moves that hold up the matrix pipeline).
    // Two tiles per trip so that each copy of the code names its buffers statically.
    auto tile_loop = [&](auto NTA_TAG) {
        constexpr int NTA = decltype(NTA_TAG)::value;
        int tile = s * P.tps;
        if (tile < t_end) issue_tile(tile, bufA);
        while (tile < t_end) {
            __builtin_amdgcn_s_waitcnt(0);     // this wave's loads have landed
            __syncthreads();                   // everyone's have, and nobody still reads bufB
            if (tile + 1 < t_end) issue_tile(tile + 1, bufB);
            wgrad_steps<NJ, NT, NTA>(acc, bufA, aoff, boff, kw, nkp, grp, P.dTX, P.TX, TXH, ntw);
            ++tile;
            if (tile >= t_end) break;
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            if (tile + 1 < t_end) issue_tile(tile + 1, bufA);
            wgrad_steps<NJ, NT, NTA>(acc, bufB, aoff, boff, kw, nkp, grp, P.dTX, P.TX, TXH, ntw);
            ++tile;
        }
    };
    if (NH == 1 || ntw == NT)
        tile_loop(std::integral_constant<int, NT>{});
    else if (NT > 1 && ntw == NT - 1)
        tile_loop(std::integral_constant<int, (NT > 1 ? NT - 1 : 1)>{});
    else
        tile_loop(std::integral_constant<int, -1>{});

    // add the accumulators of the four waves of each half in the order 0 + 1 + 2 + 3
    floatx4* red = reinterpret_cast<floatx4*>(bufA) + half * (NJ * NT * 64);
    for (int w = 1; w < 4; ++w) {
        __syncthreads();
        if (kw == w) {
#pragma unroll
            for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) red[(jt * NT + nt) * 64 + lane] = acc[jt][nt];
        }
        __syncthreads();
        if (kw == 0) {
#pragma unroll
            for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const floatx4 v = red[(jt * NT + nt) * 64 + lane];
                    acc[jt][nt] += v;
                }
        }
    }
    if (kw == 0) {
        float* out = P.partial + ((long)(s * P.AB + ab) * P.Mpad + jg * NJ * 16) * P.Npad + (cg * NH + half) * NT * 16;
#pragma unroll
        for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    out[(long)(jt * 16 + grp * 4 + r) * P.Npad + nt * 16 + col] = acc[jt][nt][r];
    }
}

// gw[j][i][a][b][c] = sum over splits of partial[s][ab][j][c*f + i], ascending s.
__global__ void __launch_bounds__(256)
k_wgrad_reduce(const float* __restrict__ partial, float* __restrict__ gw, int f, int fo, int kz, int ky, int kx,
               int ksplit, int Mpad, int Npad, int mapmajor)
{
    const int taps = kz * ky * kx;
    const long total = (long)fo * f * taps;
    const long t = (long)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const int tap = (int)(t % taps);
    const long e = t / taps;
    const int i = (int)(e % f), j = (int)(e / f);
    const int c = tap % kx, ab = tap / kx;
    const int AB = kz * ky;
    const int n = mapmajor ? i * kx + c : c * f + i;
    float acc = 0.f;
    for (int s = 0; s < ksplit; ++s) acc += partial[((long)(s * AB + ab) * Mpad + j) * Npad + n];
    gw[t] = acc;
}

using WgradFn = void (*)(WgradTile);

constexpr int kMaxTiles = 40;   // accumulator tiles per wave (4 registers each)

// Per-wave tile budget: 40 tiles with four waves (one per SIMD), 24 with eight (two per
// SIMD share the register file).
template <int NJ, int NT, int NH> WgradFn inst()
{
    if constexpr (NJ * NT <= (NH == 1 ? kMaxTiles : NH == 2 ? 24 : 12)) return k_wgrad_mfma<NJ, NT, NH>;
    else return nullptr;
}

template <int NJ, int NH> WgradFn pick_nt(int nt)
{
    switch (nt) {
        case 1: return inst<NJ, 1, NH>();
        case 2: return inst<NJ, 2, NH>();
        case 3: return inst<NJ, 3, NH>();
        case 4: return inst<NJ, 4, NH>();
        case 5: return inst<NJ, 5, NH>();
        case 6: return inst<NJ, 6, NH>();
        case 7: return inst<NJ, 7, NH>();
        case 8: return inst<NJ, 8, NH>();
        case 10: return inst<NJ, 10, NH>();
        case 13: return inst<NJ, 13, NH>();
        case 16: return inst<NJ, 16, NH>();
    }
    return nullptr;
}

template <int NH> WgradFn pick_nj(int nj, int nt)
{
    switch (nj) {
        case 1: return pick_nt<1, NH>(nt);
        case 2: return pick_nt<2, NH>(nt);
        case 3: return pick_nt<3, NH>(nt);
        case 4: return pick_nt<4, NH>(nt);
        case 5: return pick_nt<5, NH>(nt);
        case 6: return pick_nt<6, NH>(nt);
        case 7: return pick_nt<7, NH>(nt);
        case 8: return pick_nt<8, NH>(nt);
    }
    return nullptr;
}

WgradFn pick_wgrad(int nj, int nt, int nh)
{
    // sixteen waves (NH = 4) were measured slower than eight on every benchmark shape and are not instantiated
    return nh == 2 ? pick_nj<2>(nj, nt) : nh == 1 ? pick_nj<1>(nj, nt) : nullptr;
}

struct WgradChoice {
    bool ok;
    int NJ, JG, NT, G, NH;
    int TX, XT, R, GS, IS, TXH;
    int Mpad, Npad;
    int tiles, tps, ksplit;
    int vec4, fast, mapmajor;
    size_t lds;
};


// Map stride in LDS: a multiple of 4 floats (16-byte loads land on 16-byte boundaries)
// whose residue modulo 32 spreads the 16 maps of an MFMA operand over the banks.
int pad_stride(int n)
{
    static const int res = [] { const char* e = getenv("ZNN_WGRAD_STRIDE_MOD"); return e ? atoi(e) : 4; }();
    while (n % 32 != res) ++n;
    return n;
}

WgradChoice choose_wgrad(const Geom& g)
{
    WgradChoice c = {};
    c.ok = false;
    const int mt = (g.fo + 15) / 16;
    // at most six 16-map tiles per workgroup: with seven or eight the gout half of the LDS tile leaves
    // too few voxels per tile (config 5: 187 -> 160 ms with two groups of four)
    static const int maxnj = [] { const char* e = getenv("ZNN_WGRAD_MAXNJ"); const int v = e ? atoi(e) : 6; return v >= 1 && v <= 8 ? v : 6; }();
    c.JG = (mt + maxnj - 1) / maxnj;
    c.NJ = (mt + c.JG - 1) / c.JG;
    const int ncols = g.f * g.kx;
    const int nt_tot = (ncols + 15) / 16;
    const int allowed[11] = {1, 2, 3, 4, 5, 6, 7, 8, 10, 13, 16};
    int nt_max = 1;
    for (int k = 0; k < 11; ++k)
        if (c.NJ * allowed[k] <= kMaxTiles) nt_max = allowed[k];
    c.G = (nt_tot + nt_max - 1) / nt_max;
    const int want = (nt_tot + c.G - 1) / c.G;
    c.NT = nt_max;
    for (int k = 10; k >= 0; --k)
        if (allowed[k] >= want && c.NJ * allowed[k] <= kMaxTiles) c.NT = allowed[k];
    c.G = (nt_tot + c.NT - 1) / c.NT;
    // eight waves: the column tiles of a group are dealt to two halves of four waves each
    static const int halves = [] { const char* e = getenv("ZNN_WGRAD_HALVES"); return e ? atoi(e) : 2; }();
    c.NH = 1;
    for (int nh = halves; nh >= 2; nh /= 2) {
        const int nt = (c.NT + nh - 1) / nh;
        if ((nh == 2 || nh == 4) && c.NT >= nh && pick_wgrad(c.NJ, nt, nh)) {
            c.NH = nh;
            c.NT = nt;
            c.G = (nt_tot + c.NT * c.NH - 1) / (c.NT * c.NH);
            break;
        }
    }
    if (!pick_wgrad(c.NJ, c.NT, c.NH)) return c;
    c.Mpad = c.JG * c.NJ * 16;
    c.Npad = c.G * c.NT * c.NH * 16;
    // Column order.  With n = c*f + i (x-tap major) a column group spans all f input maps as soon as
    // it is wider than f, so the LDS tile of a layer with many input maps holds few voxels; with
    // n = i*kx + c (map major) a group holds only the maps of its own columns.  One group: the same
    // either way (tap major kept).  Several groups: map major.
    c.mapmajor = c.G > 1 ? 1 : 0;
    // widest x-tap span and largest input-map range over the column groups; whether every group's
    // tile starts at x-tap kx-1 (then rows of the in tile start 16-byte aligned)
    int cspan = 0, nmaps = 1;
    bool aligned_rows = true;
    for (int cg = 0; cg < c.G; ++cg) {
        const int n0 = cg * c.NT * c.NH * 16;
        const int n1 = n0 + c.NT * c.NH * 16 < ncols ? n0 + c.NT * c.NH * 16 : ncols;
        int cmin, cmax, maps;
        if (c.mapmajor) {
            const int imin = n0 / g.kx, imax = (n1 - 1) / g.kx;
            cmin = 0; cmax = g.kx - 1;
            if (imin == imax) { cmin = n0 % g.kx; cmax = (n1 - 1) % g.kx; }
            maps = imax - imin + 1;
        } else {
            cmin = n0 / g.f; cmax = (n1 - 1) / g.f;
            maps = cmax == cmin ? (n1 - 1) % g.f - n0 % g.f + 1 : g.f;
        }
        if (cmax - cmin > cspan) cspan = cmax - cmin;
        if (maps > nmaps) nmaps = maps;
        if (cmax != g.kx - 1) aligned_rows = false;
    }
    if ((size_t)c.NJ * c.NT * c.NH * 64 * 4 > (size_t)kBufFloats) return c;   // cross-wave reduction needs this
    const int rows = g.oz * g.oy;
    // fewest x-segments whose tile fits a buffer, then as many rows as fit
    for (int XT = 1; XT <= g.ox; ++XT) {
        const int seg = (g.ox + XT - 1) / XT;
        int TX = (seg + 3) & ~3;
        if (TX % 8 != 0 && rows < 2) TX += 4;          // a single row must hold whole 8-voxel steps
        const int TXH = (TX + cspan * g.spx + 3) & ~3;
        int bestR = 0;
        for (int R = 1; R <= 32 && R <= rows; ++R) {
            // the MFMA loop walks 8 voxels per step; a tile that ends on half a step reads its last four
            // voxels from the zero padding behind the row (gout) and from whatever follows (in)
            const int rtp = (R * TX + 7) & ~7;
            const long floats = (long)c.NJ * 16 * pad_stride(rtp) + (long)nmaps * pad_stride(R * TXH) + 64;
            if (floats <= kBufFloats) bestR = R;
        }
        if (bestR == 0) continue;
        c.XT = XT; c.TX = TX; c.TXH = TXH; c.R = bestR;
        c.GS = pad_stride((bestR * TX + 7) & ~7); c.IS = pad_stride(bestR * TXH);
        c.lds = 2 * (size_t)kBufFloats * 4;
        // 16-byte loads: groups of four x-neighbours must be wholly inside or outside the
        // images and start on multiples of four in both tensors
        c.vec4 = (g.ox % 4 == 0 && g.nx % 4 == 0 && aligned_rows) ? 1 : 0;
        c.ok = true;
        break;
    }
    if (!c.ok) return c;
    c.tiles = ((rows + c.R - 1) / c.R) * c.XT;
    // one workgroup per compute unit: split the voxel range until the grid reaches 256
    const long other = (long)g.kz * g.ky * c.G * c.JG;
    long ks = 256 / other;
    if (ks < 1) ks = 1;
    if (ks > c.tiles) ks = c.tiles;
    c.tps = (int)((c.tiles + ks - 1) / ks);
    c.ksplit = (c.tiles + c.tps - 1) / c.tps;
    {
        // fast tile loader: see the kernel.  Spans per wave must fit its register arrays, and a lane's
        // offset from the tile origin (up to a whole group of maps) must fit 32 bits.
        const int nw = 4 * c.NH;
        const long span_g = ((long)c.NJ * 16 * c.GS + 255) / 256, span_i = ((long)nmaps * c.IS + 255) / 256;
        c.fast = (c.vec4 && c.XT == 1 && g.oy % c.R == 0 && (span_g + nw - 1) / nw <= 5 && (span_i + nw - 1) / nw <= 5 &&
                  (double)g.fo * g.ovol() * 4.0 < 2147483648.0 && (double)g.f * g.nvol() * 4.0 < 2147483648.0 &&
                  !getenv("ZNN_WGRAD_SLOW_LOADER")) ? 1 : 0;
    }
    if ((long)g.kz * g.ky > 65535 || (long)c.G * c.JG > 65535) c.ok = false;
    // the tile loader addresses a map with a 32-bit byte offset
    if (g.nvol() >= (1L << 30) || g.ovol() >= (1L << 30)) c.ok = false;
    return c;
}

}  // namespace

bool mfma_wgrad_supported(const Geom& g) { return choose_wgrad(g).ok; }

size_t mfma_wgrad_workspace(const Geom& g)
{
    const WgradChoice c = choose_wgrad(g);
    if (!c.ok) return 0;
    return align256((size_t)c.ksplit * g.kz * g.ky * c.Mpad * c.Npad * sizeof(float));
}

int mfma_wgrad(const Geom& g, const float* in, const float* gout, float* gw, void* ws, hipStream_t s)
{
    const WgradChoice c = choose_wgrad(g);
    if (!c.ok) return fail(ZNN_EUNSUPPORTED, "no tile configuration fits this shape");
    WgradTile P = {};
    P.in = in; P.gout = gout; P.partial = (float*)ws;
    P.f = g.f; P.fo = g.fo;
    P.nz = g.nz; P.ny = g.ny; P.nx = g.nx;
    P.oz = g.oz; P.oy = g.oy; P.ox = g.ox;
    P.kz = g.kz; P.ky = g.ky; P.kx = g.kx;
    P.spz = g.spz; P.spy = g.spy; P.spx = g.spx;
    P.TX = c.TX; P.XT = c.XT; P.R = c.R;
    P.GS = c.GS; P.IS = c.IS; P.TXH = c.TXH;
    P.Mpad = c.Mpad; P.Npad = c.Npad;
    P.G = c.G;
    P.tiles = c.tiles; P.tps = c.tps;
    P.AB = g.kz * g.ky;
    P.vec4 = c.vec4;
    P.fast = c.fast;
    P.mapmajor = c.mapmajor;
    P.dGS = make_fastdiv(c.GS); P.dIS = make_fastdiv(c.IS);
    P.dTX = make_fastdiv(c.TX); P.dTXH = make_fastdiv(c.TXH); P.dOY = make_fastdiv(g.oy);
    if (log_enabled())
        fprintf(stderr, "[znn] wgrad mfma: NJ=%d JG=%d NT=%d NH=%d G=%d TX=%d XT=%d R=%d lds=%zu ksplit=%d tiles=%d\n",
                c.NJ, c.JG, c.NT, c.NH, c.G, c.TX, c.XT, c.R, c.lds, c.ksplit, c.tiles);
    WgradFn fn = pick_wgrad(c.NJ, c.NT, c.NH);
    if (!fn) return fail(ZNN_EUNSUPPORTED, "no kernel instance for tile %dx%d", c.NJ, c.NT);
    ZNN_LAUNCH("direct kernel gradient (MFMA)", s, fn, dim3((unsigned)c.ksplit, (unsigned)P.AB, (unsigned)(c.G * c.JG)), dim3(256 * c.NH), 0, P);
    int rc = check_launch("direct kernel gradient (MFMA)");
    if (rc != ZNN_OK) return rc;
    const long total = (long)g.fo * g.f * g.kvol();
    ZNN_LAUNCH("kernel gradient reduction", s, k_wgrad_reduce, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       (const float*)ws, gw, g.f, g.fo, g.kz, g.ky, g.kx, c.ksplit, c.Mpad, c.Npad, c.mapmajor);
    return check_launch("kernel gradient reduction");
}

}  // namespace znn
