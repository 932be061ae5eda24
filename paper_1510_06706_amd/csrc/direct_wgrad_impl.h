// Kernel of the direct method's kernel gradient on the fp32 matrix cores, shared by the
// translation units that instantiate it (one per wave count); the host side is in
// direct_wgrad_mfma.hip, which also describes the algorithm.
#pragma once

#include <type_traits>

#include "znn_internal.h"

namespace znn {
namespace wgrad {


typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) const void* global_cptr;
typedef __attribute__((address_space(3))) void* lds_ptr;

// Two tile buffers as separate LDS objects: the compiler then knows that loads
// landing in one buffer do not alias reads of the other and lets them overlap.
constexpr int kBufFloats = 18432;                 // 72 KiB each

// Spans of 256 floats of a tile region that one wave of the fast loader may have to fetch (one offset
// register each): either region can take nearly the whole buffer (72 spans), dealt over the workgroup's
// waves.  Eight-wave kernels with at most three map tiles keep the five that their tiles have needed so
// far (the longer unrolled loader costs them 3 %).
constexpr int max_spans(int waves, int nj) { return waves >= 8 ? (nj <= 3 ? 5 : 9) : 18; }

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
// two-dword LDS read and feeds two MFMAs from it.  The wave takes steps kp, kp+KW, ... < k1.
// Two register sets take turns, so the LDS reads of the next step are queued before the
// MFMAs of the current one and only waited for after them; the code is kept free of
// branches around loads and MFMAs (a step past the end re-reads the last one, NTA is the
// compile-time number of column tiles that hold real columns) because the compiler can
// only count outstanding loads exactly in straight-line code.  NTA < 0: the number of
// live tiles is the run-time value ntw (any ragged column group; slower).
template <int NJ, int NT, int NTA, int KW>
__device__ __forceinline__ void wgrad_steps(floatx4 (&acc)[NJ][NT], const float* buf, const int (&aoff)[NJ],
                                            const int (&boff)[NT], int kp, int k1, int grp, FastDiv dTX, int TX,
                                            int TXH, int ntw)
{
    if (kp >= k1) return;
    const int klast = kp + ((k1 - 1 - kp) / KW) * KW;
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
        load_step(min(kp + KW, klast), a1, b1);
        mfma_step(a0, b0);
        if (kp + KW >= k1) break;
        load_step(min(kp + 2 * KW, klast), a0, b0);
        mfma_step(a1, b1);
        if (kp + 2 * KW >= k1) break;
        kp += 2 * KW;
    }
}

// The NG * KW waves of a workgroup form NG sets of KW waves: set h owns the column tiles
// [h * NT, (h + 1) * NT) of the workgroup's column group, and the KW waves of a set split the voxel
// steps of every staged tile (their accumulators are added at the end).
//   NG = 1, KW = 4   four waves share every column tile (few columns in all).
//   NG = 2, KW = 4   eight waves, two per SIMD: while one waits for its global->LDS loads to be queued
//                    the other keeps the matrix cores busy.
//   NG = 4, KW = 1   four waves with their own columns each: the workgroup covers four times the
//                    columns with the same accumulator budget per wave, so every staged gout voxel
//                    feeds four times the MFMAs (layers with many columns, where the fetch of the
//                    tiles would otherwise take as long as their MFMAs).
template <int NJ, int NT, int NG, int KW>
__global__ void __launch_bounds__(64 * NG * KW) k_wgrad_mfma(WgradTile P)
{
    constexpr int NH = NG;
    constexpr int NW = NG * KW;
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
    const int half = wave / KW, kw = wave % KW;
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
    // Lanes of a tile that lie outside the images hold zeros: the buffers are zeroed once and such lanes are
    // never loaded.  A lane that was inside for the tile this buffer held before and is outside now (tiles
    // behind the last voxel row; the last, shorter x-segment of a row) has to be zeroed by hand: `zero_pass`
    // does only that, BEFORE the tile's loads are queued, so that the LDS stores never wait for a load that
    // is still in flight (a store queued behind a load into the same buffer would wait for it to land, one
    // full memory latency per map).
    auto issue_part = [&](float* dst, int stride, const float* base, long mapvol, int nm, int width, int total,
                          FastDiv dw, int rho0, int xg0, int xlim, bool is_in, bool zero_pass, auto WT) __attribute__((always_inline)) {
        constexpr int W = decltype(WT)::value;
        for (int k = 0; k * 64 * W < total; ++k) {
            const int e = k * 64 * W + lane * W;
            const int r = (int)fdiv((unsigned)e, dw), x = e - r * width;
            const int rho = rho0 + r, gx = xg0 + x;
            const bool inside = e < total;
            const bool ok = inside && rho < rows && gx < xlim;
            if (zero_pass) {
                const bool fix = inside && !ok;
                if (__builtin_amdgcn_ballot_w64(fix) == 0) continue;       // wave-uniform
                for (int m = wave; m < nm; m += NW) {
                    float* row = dst + m * stride + k * 64 * W;             // uniform
                    if (fix) {
#pragma unroll
                        for (int q = 0; q < W; ++q) row[lane * W + q] = 0.f;
                    }
                }
                continue;
            }
            unsigned voff;
            if (is_in) {
                const int z = (int)fdiv((unsigned)rho, P.dOY), y = rho - z * P.oy;
                voff = (unsigned)((z + (P.kz - 1 - a) * P.spz) * (int)iplane + (y + (P.ky - 1 - b) * P.spy) * P.nx + gx) * 4u;
            } else {
                voff = (unsigned)(rho * P.ox + gx) * 4u;
            }
            for (int m = wave; m < nm; m += NW) {
                const char* mb = reinterpret_cast<const char*>(base + (long)m * mapvol);   // uniform
                float* row = dst + m * stride + k * 64 * W;                                 // uniform
                if (ok) {
                    if constexpr (W == 4) __builtin_amdgcn_global_load_lds((global_cptr)(mb + voff), (lds_ptr)row, 16, 0, 0);
                    else __builtin_amdgcn_global_load_lds((global_cptr)(mb + voff), (lds_ptr)row, 4, 0, 0);
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
    constexpr int kMaxSpans = max_spans(NW, NJ);
    unsigned fg_off[kMaxSpans], fi_off[kMaxSpans];
    unsigned fg_ok = 0, fi_ok = 0;          // bit q: span q of this wave holds data for this lane
    const int nspan_g = (mreal * P.GS + 255) >> 8, nspan_i = (nmaps * P.IS + 255) >> 8;
    if (P.fast) {
#pragma unroll
        for (int q = 0; q < kMaxSpans; ++q) {
            const int L = (wave + q * NW) * 256 + lane * 4;
            {
                const int m = (int)fdiv((unsigned)L, P.dGS), e = L - m * P.GS;
                const int r = (int)fdiv((unsigned)e, P.dTX), x = e - r * P.TX;
                fg_ok |= (m < mreal && e < RT && x < P.ox ? 1u : 0u) << q;
                fg_off[q] = (unsigned)(m * (int)oplane + r * P.ox + x) * 4u;
            }
            {
                const int m = (int)fdiv((unsigned)L, P.dIS), e = L - m * P.IS;
                const int r = (int)fdiv((unsigned)e, P.dTXH), x = e - r * TXH;
                const int ix = (P.kx - 1 - cmax) * P.spx + x;
                fi_ok |= (m < nmaps && e < RTH && ix < P.nx ? 1u : 0u) << q;
                fi_off[q] = (unsigned)(m * (int)ivol + r * P.nx + ix) * 4u;
            }
        }
    }
    auto issue_tile_fast = [&](int tile, float* buf) __attribute__((always_inline)) {
        const int rho0 = tile * P.R;                                    // XT == 1
        const int z = (int)fdiv((unsigned)rho0, P.dOY), y = rho0 - z * P.oy;
        const char* gb = reinterpret_cast<const char*>(P.gout + (long)(jg * NJ * 16) * oplane + (long)rho0 * P.ox);
        const char* ib = reinterpret_cast<const char*>(P.in + (long)imin * ivol + (long)(z + (P.kz - 1 - a) * P.spz) * iplane +
                                                       (long)(y + (P.ky - 1 - b) * P.spy) * P.nx);
#pragma unroll
        for (int q = 0; q < kMaxSpans; ++q) {
            const int sp = wave + q * NW;                               // uniform
            if (sp < nspan_g && (fg_ok >> q & 1u))
                __builtin_amdgcn_global_load_lds((global_cptr)(gb + fg_off[q]), (lds_ptr)(buf + sp * 256), 16, 0, 0);
        }
#pragma unroll
        for (int q = 0; q < kMaxSpans; ++q) {
            const int sp = wave + q * NW;
            if (sp < nspan_i && (fi_ok >> q & 1u))
                __builtin_amdgcn_global_load_lds((global_cptr)(ib + fi_off[q]), (lds_ptr)(buf + itoff + sp * 256), 16, 0, 0);
        }
    };
    auto issue_tile = [&](int tile, float* buf) __attribute__((always_inline)) {
        if (P.fast) { issue_tile_fast(tile, buf); return; }
        const int xt = tile % P.XT, rt = tile / P.XT;
        const int rho0 = rt * P.R, xs0 = xt * P.TX;
        const int xin0 = xs0 + (P.kx - 1 - cmax) * P.spx;
        const float* gbase = P.gout + (long)(jg * NJ * 16) * oplane;
        const float* ibase = P.in + (long)imin * ivol;
        // which lanes are inside the images is the same for every tile except those behind the last voxel row
        // and the last x-segment of a row when there are several: only those tiles need the zeroing pass
        const bool zero_first = rho0 + P.R > rows || (P.XT > 1 && xt == P.XT - 1);
        for (int pass = zero_first ? 0 : 1; pass < 2; ++pass) {
            const bool zp = pass == 0;
            if (P.vec4) {
                issue_part(buf, P.GS, gbase, oplane, mreal, P.TX, RT, P.dTX, rho0, xs0, P.ox, false, zp, std::integral_constant<int, 4>{});
                issue_part(buf + itoff, P.IS, ibase, ivol, nmaps, TXH, RTH, P.dTXH, rho0, xin0, P.nx, true, zp, std::integral_constant<int, 4>{});
            } else {
                issue_part(buf, P.GS, gbase, oplane, mreal, P.TX, RT, P.dTX, rho0, xs0, P.ox, false, zp, std::integral_constant<int, 1>{});
                issue_part(buf + itoff, P.IS, ibase, ivol, nmaps, TXH, RTH, P.dTXH, rho0, xin0, P.nx, true, zp, std::integral_constant<int, 1>{});
            }
        }
    };

    // The whole tile loop is instantiated once per variant of the MFMA steps (all column tiles
    // live, one padded tile skipped, run-time count) and the variant is chosen once, out here:
    // choosing per tile would merge the variants' register assignments after every tile, which
    // costs a copy of every accumulator (vector moves that hold up the matrix pipeline).
    // Two tiles per trip so that each copy of the code names its buffers statically.
    auto tile_loop = [&](auto NTA_TAG) __attribute__((always_inline)) {
        constexpr int NTA = decltype(NTA_TAG)::value;
        int tile = s * P.tps;
        if (tile < t_end) issue_tile(tile, bufA);
        while (tile < t_end) {
            __builtin_amdgcn_s_waitcnt(0);     // this wave's loads have landed
            __syncthreads();                   // everyone's have, and nobody still reads bufB
            if (tile + 1 < t_end) issue_tile(tile + 1, bufB);
            wgrad_steps<NJ, NT, NTA, KW>(acc, bufA, aoff, boff, kw, nkp, grp, P.dTX, P.TX, TXH, ntw);
            ++tile;
            if (tile >= t_end) break;
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            if (tile + 1 < t_end) issue_tile(tile + 1, bufA);
            wgrad_steps<NJ, NT, NTA, KW>(acc, bufB, aoff, boff, kw, nkp, grp, P.dTX, P.TX, TXH, ntw);
            ++tile;
        }
    };
    if (NH == 1 || ntw == NT)
        tile_loop(std::integral_constant<int, NT>{});
    else if (NT > 1 && ntw == NT - 1)
        tile_loop(std::integral_constant<int, (NT > 1 ? NT - 1 : 1)>{});
    else
        tile_loop(std::integral_constant<int, -1>{});

    // add the accumulators of the KW waves of each set in the order 0 + 1 + 2 + ...
    floatx4* red = reinterpret_cast<floatx4*>(bufA) + half * (NJ * NT * 64);
    for (int w = 1; w < KW; ++w) {
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

using WgradFn = void (*)(WgradTile);

constexpr int kMaxTiles = 40;   // accumulator tiles per wave (4 registers each)

// Per-wave tile budget: 40 tiles with four waves (one per SIMD), 24 with eight (two per
// SIMD share the register file).
template <int NJ, int NT, int NG, int KW> WgradFn inst()
{
    if constexpr (NJ * NT <= (NG * KW == 4 ? kMaxTiles : 24)) return k_wgrad_mfma<NJ, NT, NG, KW>;
    else return nullptr;
}

template <int NJ, int NG, int KW> WgradFn pick_nt(int nt)
{
    switch (nt) {
        case 1: return inst<NJ, 1, NG, KW>();
        case 2: return inst<NJ, 2, NG, KW>();
        case 3: return inst<NJ, 3, NG, KW>();
        case 4: return inst<NJ, 4, NG, KW>();
        case 5: return inst<NJ, 5, NG, KW>();
        case 6: return inst<NJ, 6, NG, KW>();
        case 7: return inst<NJ, 7, NG, KW>();
        case 8: return inst<NJ, 8, NG, KW>();
        case 10: return inst<NJ, 10, NG, KW>();
        case 13: return inst<NJ, 13, NG, KW>();
        case 16: return inst<NJ, 16, NG, KW>();
    }
    return nullptr;
}

// LO: one to four map tiles per workgroup, !LO: five to eight (two translation units per wave layout).
template <int NG, int KW, bool LO> WgradFn pick_nj(int nj, int nt)
{
    if constexpr (LO) {
        switch (nj) {
            case 1: return pick_nt<1, NG, KW>(nt);
            case 2: return pick_nt<2, NG, KW>(nt);
            case 3: return pick_nt<3, NG, KW>(nt);
            case 4: return pick_nt<4, NG, KW>(nt);
        }
    } else {
        switch (nj) {
            case 5: return pick_nt<5, NG, KW>(nt);
            case 6: return pick_nt<6, NG, KW>(nt);
            case 7: return pick_nt<7, NG, KW>(nt);
            case 8: return pick_nt<8, NG, KW>(nt);
        }
    }
    return nullptr;
}

}  // namespace wgrad

// One definition per translation unit direct_wgrad_{h1,h2,n4}{a,b}.hip.
wgrad::WgradFn wgrad_kernel_h1a(int nj, int nt);
wgrad::WgradFn wgrad_kernel_h1b(int nj, int nt);
wgrad::WgradFn wgrad_kernel_h2a(int nj, int nt);
wgrad::WgradFn wgrad_kernel_h2b(int nj, int nt);
wgrad::WgradFn wgrad_kernel_n4a(int nj, int nt);
wgrad::WgradFn wgrad_kernel_n4b(int nj, int nt);
wgrad::WgradFn wgrad_kernel_n8a(int nj, int nt);
wgrad::WgradFn wgrad_kernel_n8b(int nj, int nt);

}  // namespace znn
