// Kernel of the direct method's forward and backward pass (see direct_mfma_impl.h for the tile scheme and
// the tap loop), shared by the translation units that instantiate it for one x-tap group width each.
//
//   full 16-map tiles      v_mfma_f32_16x16x4_f32       m: 16 maps, n: 16 voxels, k: the chunk's 4 input maps
//   the last 1..8 maps of  v_mfma_f32_4x4x1_16B_f32     16 independent 4x4 outer products per instruction:
//   a count 16 q + r,                                   block (mt, nt) = 4 maps x 4 voxels, mt < 2, nt < 8,
//   r <= 8 (TAIL)                                       i.e. 8 maps x 32 voxels (two voxel tiles) and ONE
//                                                       input map; four instructions cover the chunk
//
// Both forms run at the same peak rate per multiply-add, so the eight maps cost 8/16 of a padded
// tile (40, 88, 120 maps: no padding left).  What the second form needs: its B operand holds for lane
// (block, v) the voxel nt*4 + v of one input map, its A operand for lane (block, m) the weight of map
// mt*4 + m.  The halo box is therefore staged with the chunk's four maps interleaved, word = 4 * voxel + map:
// a lane gets the four maps of its voxel with one 16-byte LDS read (one register per instruction), and the
// 16x16x4 operand (lane = map * 16 + voxel) reads 64 consecutive words for 16 consecutive voxels, which
// spreads over the LDS banks whatever the box (a map-major box needs a stride that keeps the four maps
// apart in the banks and still collided; layers of full tiles only gained 9 % from the change of layout
// alone).  The packed weights carry, behind the full tiles of every tap, 8 maps x 4 input maps for the
// same kind of read.
#pragma once

#include "direct_mfma_impl.h"

namespace znn {
namespace conv {

// LDS addresses are kept as 32-bit LDS pointers that already include the buffer's base, so an operand
// read is one ds_read with an immediate offset and a tap group costs one vector addition per operand.
typedef __attribute__((address_space(3))) const char* lds_bytes;
typedef __attribute__((address_space(3))) const float* lds_floatp;
typedef __attribute__((address_space(3))) const floatx4* lds_float4p;

constexpr int kTailMaps = 8;
constexpr int kTailPacked = kTailMaps * 4;      // floats behind the full tiles of a tap

// One tap: the MFMAs of the current operand set with the LDS reads of the next tap's 16x16x4 operands
// dealt between them.  The 4x4x1 voxel operands `bt` of THIS tap were requested just before the call
// and arrive while the full tiles run.
template <int NJ, int NV, int NP>
__device__ __forceinline__ void tap_mfmas_tail(floatx4 (&acc)[NJ][NV], floatx4 (&accT)[NP ? NP : 1], const float (&a)[NJ],
                                               const float (&b)[NV], const floatx4& at, const floatx4 (&bt)[NP ? NP : 1],
                                               float (&bn)[NV], const lds_bytes (&vb)[NV], int imm)
{
#pragma unroll
    for (int jt = 0; jt < NJ; ++jt) {
#pragma unroll
        for (int nv = 0; nv < NV; ++nv) acc[jt][nv] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[jt], b[nv], acc[jt][nv], 0, 0, 0);
#pragma unroll
        for (int nv = jt * NV / NJ; nv < (jt + 1) * NV / NJ; ++nv) bn[nv] = *reinterpret_cast<lds_floatp>(vb[nv] + imm * 16);
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int pr = 0; pr < NP; ++pr) accT[pr] = __builtin_amdgcn_mfma_f32_4x4x1f32(at[k], bt[pr][k], accT[pr], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
}

// The U taps of one group (see group_step in direct_mfma_impl.h).  wlo: the lane's index into the
// group's full-tile weights, wto: into its 8-map block (LDS copy of the chunk's weights when WL; else
// the packed weights are read from global memory at wg, the group's first tap).
template <int NJ, int NV, int NP, bool WL, int U, int PAR>
__device__ __forceinline__ void group_step_tail(floatx4 (&acc)[NJ][NV], floatx4 (&accT)[NP ? NP : 1], float (&a0)[NJ],
                                                float (&b0)[NV], floatx4& at0, float (&a1)[NJ], float (&b1)[NV],
                                                floatx4& at1, lds_bytes (&vb)[NV], lds_bytes (&vbT)[NP ? NP : 1],
                                                const lds_bytes (&voff)[NV], const lds_bytes (&voffT)[NP ? NP : 1],
                                                const float*& wg, const float* wl, int& wlo, int& wto, unsigned lane,
                                                unsigned tl4, int o_next, int advance)
{
    constexpr bool TAIL = NP > 0;
    constexpr int WT = NJ * 64 + (TAIL ? kTailPacked : 0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const bool odd = ((PAR + u) & 1) != 0;
        float (&ac)[NJ] = odd ? a1 : a0;
        float (&bc)[NV] = odd ? b1 : b0;
        floatx4& atc = odd ? at1 : at0;
        float (&an)[NJ] = odd ? a0 : a1;
        float (&bn)[NV] = odd ? b0 : b1;
        floatx4& atn = odd ? at0 : at1;
        floatx4 bt[NP ? NP : 1];
#pragma unroll
        for (int pr = 0; pr < NP; ++pr) bt[pr] = *reinterpret_cast<lds_float4p>(vbT[pr] + (U - 1 - u) * 16);
        if (u + 1 < U) {
            const float* wtap = wg + (u + 1) * WT;      // uniform
#pragma unroll
            for (int jt = 0; jt < NJ; ++jt) an[jt] = WL ? wl[wlo + (u + 1) * WT + jt * 64] : wtap[jt * 64 + lane];
            if constexpr (TAIL)
                atn = WL ? *reinterpret_cast<const floatx4*>(wl + wto + (u + 1) * WT)
                         : *reinterpret_cast<const floatx4*>(wtap + NJ * 64 + tl4);
            __builtin_amdgcn_sched_barrier(0);
            tap_mfmas_tail<NJ, NV, NP>(acc, accT, ac, bc, atc, bt, bn, vb, U - 2 - u);
        } else {
            if (advance) {      // floats to the next group's packed weights, 0 after the last group
                wg += advance;
                if (WL) { wlo += advance; wto += advance; }
            }
#pragma unroll
            for (int nv = 0; nv < NV; ++nv) vb[nv] = voff[nv] + o_next * 16;
#pragma unroll
            for (int jt = 0; jt < NJ; ++jt) an[jt] = WL ? wl[wlo + jt * 64] : wg[jt * 64 + lane];
            if constexpr (TAIL)
                atn = WL ? *reinterpret_cast<const floatx4*>(wl + wto) : *reinterpret_cast<const floatx4*>(wg + NJ * 64 + tl4);
            __builtin_amdgcn_sched_barrier(0);
            tap_mfmas_tail<NJ, NV, NP>(acc, accT, ac, bc, atc, bt, bn, vb, U - 1);
#pragma unroll
            for (int pr = 0; pr < NP; ++pr) vbT[pr] = voffT[pr] + o_next * 16;
        }
    }
}

// NJ full 16-map tiles, plus the 8-map block when TAIL; NV voxel tiles per wave.  P.MS is the halo box
// rounded up to 16 voxels; a halo buffer holds 4 * P.MS words.  Without the block, gridDim.y groups of
// NJ tiles cover more than 128 maps.
template <int NJ, int NV, bool WL, int U, bool TAIL>
__global__ void __launch_bounds__(256, 2) k_conv_mfma_tail(ConvTile P)
{
    constexpr int NP = TAIL ? (NV + 1) / 2 : 0;
    constexpr int NPA = NP ? NP : 1;
    constexpr int WT = NJ * 64 + (TAIL ? kTailPacked : 0);
    extern __shared__ __attribute__((aligned(16))) float lds4[];
    float* lds = lds4;
    const int taps = P.kz * P.ky * P.kx;
    const int MSP = (P.MS + 255) & ~255;
    const int nbuf = P.dbuf ? 2 : 1;
    int* tab = reinterpret_cast<int*>(lds + nbuf * 4 * P.MS);
    float* wl = lds + nbuf * 4 * P.MS + MSP;
    const unsigned lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = lane & 15, grp = lane >> 4;
    // the lane's place in the 4x4x1 operands: block = lane / 4 = (mt, nt), element = lane % 4
    const unsigned tl = (lane >> 5) * 4 + (lane & 3);   // map of the 8-map block this lane holds a weight of
    const int tv32 = ((lane >> 2) & 7) * 4 + (lane & 3);    // voxel of the 32-voxel pair this lane holds

    int b = blockIdx.x;
    const int bxi = b % P.cx; b /= P.cx;
    const int byi = b % P.cy;
    const int bzi = b / P.cy;
    const int z0 = bzi * P.Tz, y0 = byi * P.Ty, x0 = bxi * P.Tx;
    const int Ttot = P.Tz * P.Ty * P.Tx;

    // byte offsets of the lane's voxels in a halo buffer (a voxel is four words, one per map).  With an odd
    // number of voxel tiles the upper half of the last pair is idle: it reads voxel 0 and stores nothing.
    auto halo_byte = [&](int t) {
        if (t >= Ttot) t = 0;
        const int tx = t % P.Tx, ty = (t / P.Tx) % P.Ty, tz = t / (P.Tx * P.Ty);
        return ((tz * P.HY + ty) * P.HX + tx) * 16;
    };
    auto pair_live = [&](int pr) { return 2 * pr + 1 < NV || tv32 < 16; };
    const lds_bytes lbase = (lds_bytes)lds;
    lds_bytes voff[NV], voffT[NPA];
#pragma unroll
    for (int nv = 0; nv < NV; ++nv) voff[nv] = lbase + (halo_byte((wave * NV + nv) * 16 + col) + grp * 4);
#pragma unroll
    for (int pr = 0; pr < NP; ++pr) voffT[pr] = lbase + (pair_live(pr) ? halo_byte((wave * NV + 2 * pr) * 16 + tv32) : 0);

    floatx4 acc[NJ][NV], accT[NPA];
#pragma unroll
    for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
        for (int nv = 0; nv < NV; ++nv) acc[jt][nv] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int pr = 0; pr < NP; ++pr) accT[pr] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int hvol = P.HZ * P.HY * P.HX;
    const long splane = (long)P.sy * P.sx;
    const long svol = (long)P.sz * splane;
    const int ic0 = blockIdx.z * P.cps, ic1 = min(P.nchunk, ic0 + P.cps);
    const int jg = blockIdx.y;
    const float* wq = P.wp + ((long)jg * P.nchunk + ic0) * taps * WT;      // uniform
    const int groups_per_row = P.kx / U;
    // planes and rows of taps that meet the source somewhere in this workgroup's box (all of them unless the
    // box lies in the zero-extended border of the backward pass)
    int alo, ahi, blo, bhi;
    live_taps(z0, min(P.Tz, P.dz - z0), P.pz, P.sz, P.kz, P.spz, alo, ahi);
    live_taps(y0, min(P.Ty, P.dy - y0), P.py, P.sy, P.ky, P.spy, blo, bhi);
    const bool none = ahi < alo || bhi < blo;
    if (none) { alo = ahi = 0; blo = bhi = 0; }
    const int na = ahi - alo + 1, nb = bhi - blo + 1;
    const int ngroups = none ? 0 : na * nb * groups_per_row;
    const int wstart = ((P.kz - 1 - ahi) * P.ky + (P.ky - 1 - bhi)) * P.kx * WT;    // first packed tap of the walk
    const int wrow = (P.ky - nb) * P.kx * WT;

    // Halo loader: tab[r] = byte offset inside a source map of voxel r of the halo box, -1 outside the
    // image (zero padding) and behind the box.  A wave-load fills 64 consecutive words = 16 voxels x
    // 4 maps: lane l fetches voxel l / 4 of map l % 4.
    if (P.nchunk < 0) lds[threadIdx.x] = P.src[threadIdx.x];    // never taken: tells the optimizer that LDS holds data
    for (int r = threadIdx.x; r < MSP; r += 256) {
        int v = -1;
        if (r < hvol) {
            const int r1 = (int)fdiv((unsigned)r, P.dHX), hx = r - r1 * P.HX;
            const int hz = (int)fdiv((unsigned)r1, P.dHY), hy = r1 - hz * P.HY;
            const int gz = z0 + hz - P.pz, gy = y0 + hy - P.py, gx = x0 + hx - P.px;
            if (gz >= 0 && gz < P.sz && gy >= 0 && gy < P.sy && gx >= 0 && gx < P.sx)
                v = ((gz * P.sy + gy) * P.sx + gx) * 4;
        }
        tab[r] = v;
    }
    for (int q = threadIdx.x; q < nbuf * 4 * P.MS; q += 256) lds[q] = 0.f;
    __syncthreads();

    const int kmap = lane & 3;
    const unsigned kofs = (unsigned)kmap * (unsigned)(svol * 4);    // the host admits only 16 * svol < 2^32
    const int nspan = P.MS >> 4;
    auto issue_chunk = [&](int ic, float* buf) {
        const int nvalid = min(4, P.fK - ic * 4);
        const char* cb = reinterpret_cast<const char*>(P.src + (long)ic * 4 * svol);    // uniform
        if (nvalid < 4)     // last chunk of a fan-in that is no multiple of four: the missing maps read as zero
            for (int q = threadIdx.x; q < 4 * P.MS; q += 256)
                if ((q & 3) >= nvalid) buf[q] = 0.f;
        for (int q0 = wave; q0 < nspan; q0 += 16) {
            int tv[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) tv[j] = q0 + 4 * j < nspan ? tab[(q0 + 4 * j) * 16 + (lane >> 2)] : -1;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int q = q0 + 4 * j;       // uniform
                if (q < nspan && tv[j] >= 0 && kmap < nvalid)
                    __builtin_amdgcn_global_load_lds((global_cptr)(cb + ((unsigned)tv[j] + kofs)), (lds_ptr)(buf + q * 64), 4, 0, 0);
            }
        }
    };

    if (P.dbuf && ic0 < ic1) issue_chunk(ic0, lds);
    for (int ic = ic0; ic < ic1; ++ic) {
        const int cur = P.dbuf ? (ic - ic0) & 1 : 0;
        if (!P.dbuf) {
            __syncthreads();
            issue_chunk(ic, lds);
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (WL) {
            const floatx4* src4 = reinterpret_cast<const floatx4*>(wq);
            floatx4* dst4 = reinterpret_cast<floatx4*>(wl);
            for (int t = threadIdx.x; t < taps * (WT / 4); t += 256) dst4[t] = src4[t];
            __syncthreads();
        }
        if (P.dbuf && ic + 1 < ic1) issue_chunk(ic + 1, lds + (cur ^ 1) * 4 * P.MS);

        float a0[NJ], b0[NV], a1[NJ], b1[NV];
        floatx4 at0, at1;
        lds_bytes vb[NV], vbT[NPA];
        GroupWalk<U> walk;
        walk.start(P, ahi, bhi, nb, wrow);
        walk.o += cur * P.MS;               // in voxels; a voxel is four words
        const float* wg = wq + wstart;
        int wlo = lane + wstart, wto = NJ * 64 + tl * 4 + wstart;
        const unsigned tl4 = tl * 4;
#pragma unroll
        for (int nv = 0; nv < NV; ++nv) vb[nv] = voff[nv] + walk.o * 16;
#pragma unroll
        for (int pr = 0; pr < NP; ++pr) vbT[pr] = voffT[pr] + walk.o * 16;
#pragma unroll
        for (int jt = 0; jt < NJ; ++jt) a0[jt] = WL ? wl[wlo + jt * 64] : wg[jt * 64 + lane];
        if constexpr (TAIL)
            at0 = WL ? *reinterpret_cast<const floatx4*>(wl + wto) : *reinterpret_cast<const floatx4*>(wg + NJ * 64 + tl4);
        else
            at0 = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int nv = 0; nv < NV; ++nv) b0[nv] = *reinterpret_cast<lds_floatp>(vb[nv] + (U - 1) * 16);
        at1 = at0;

        int g = 0;
        for (; g + 2 <= ngroups; g += 2) {
            int wd = U * WT;
            walk.o += walk.step(P, groups_per_row, wd);
            group_step_tail<NJ, NV, NP, WL, U, 0>(acc, accT, a0, b0, at0, a1, b1, at1, vb, vbT, voff, voffT, wg, wl, wlo,
                                              wto, lane, tl4, walk.o, wd);
            const bool more = g + 2 < ngroups;
            wd = more ? U * WT : 0;
            if (more) walk.o += walk.step(P, groups_per_row, wd);
            group_step_tail<NJ, NV, NP, WL, U, (U & 1)>(acc, accT, a0, b0, at0, a1, b1, at1, vb, vbT, voff, voffT, wg, wl,
                                                    wlo, wto, lane, tl4, walk.o, wd);
            asm volatile("" ::: "memory");
        }
        if (g < ngroups)
            group_step_tail<NJ, NV, NP, WL, U, 0>(acc, accT, a0, b0, at0, a1, b1, at1, vb, vbT, voff, voffT, wg, wl, wlo,
                                              wto, lane, tl4, walk.o, 0);
        wq += (long)taps * WT;
    }

    const long dplane = (long)P.dy * P.dx;
    const long dvol = (long)P.dz * dplane;
    float* out = gridDim.z > 1 ? P.partial + (long)blockIdx.z * P.fM * dvol : P.dst;
    auto voxel_of = [&](int t) -> long {
        if (t >= Ttot) return -1;
        const int tx = t % P.Tx, ty = (t / P.Tx) % P.Ty, tz = t / (P.Tx * P.Ty);
        const int z = z0 + tz, y = y0 + ty, x = x0 + tx;
        if (z >= P.dz || y >= P.dy || x >= P.dx) return -1;
        return z * dplane + (long)y * P.dx + x;
    };
    // 16x16x4: lane holds rows m = 4*(lane/16) + r, column n = lane%16
#pragma unroll
    for (int nv = 0; nv < NV; ++nv) {
        const long vox = voxel_of((wave * NV + nv) * 16 + col);
        if (vox < 0) continue;
#pragma unroll
        for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int j = (jg * NJ + jt) * 16 + grp * 4 + r;
                if (TAIL || j < P.fM) out[(long)j * dvol + vox] = acc[jt][nv][r];
            }
    }
    // 4x4x1: lane (block (mt, nt), v) holds maps mt*4 + r of voxel nt*4 + v
#pragma unroll
    for (int pr = 0; pr < NP; ++pr) {
        const long vox = pair_live(pr) ? voxel_of((wave * NV + 2 * pr) * 16 + tv32) : -1;
        if (vox < 0) continue;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int j = NJ * 16 + (lane >> 5) * 4 + r;
            if (j < P.fM) out[(long)j * dvol + vox] = accT[pr][r];
        }
    }
}

// Instances.  With the block: 1..7 full tiles, 4 to 8 voxel tiles per wave, at most 28 accumulator tiles (more
// spill registers at two workgroups per compute unit; so does 4 x 7, whose four partial sums of the block come
// on top of the 28 tiles: 35 registers spilled).  Without: 1..8 tiles, 2 or 4..8 voxel tiles, at most 32.
constexpr bool tail_instance(int nj, int nv)
{
    return nj >= 1 && nj <= 7 && nv >= 4 && nv <= 8 && nj * nv <= 28 && !(nj == 4 && nv == 7);
}
constexpr bool plain_instance(int nj, int nv)
{
    return nj >= 1 && nj <= 8 && (nv == 2 || (nv >= 4 && nv <= 8)) && (nv <= 4 || nj * nv <= 32);
}

template <int NJ, int NV, bool WL, int U, bool TAIL> ConvFn conv_instance()
{
    if constexpr (TAIL ? tail_instance(NJ, NV) : plain_instance(NJ, NV)) return k_conv_mfma_tail<NJ, NV, WL, U, TAIL>;
    else return nullptr;
}

template <int NJ, bool WL, int U, bool TAIL> ConvFn pick_tail_nv(int nv)
{
    switch (nv) {
        case 2: return conv_instance<NJ, 2, WL, U, TAIL>();
        case 4: return conv_instance<NJ, 4, WL, U, TAIL>();
        case 5: return conv_instance<NJ, 5, WL, U, TAIL>();
        case 6: return conv_instance<NJ, 6, WL, U, TAIL>();
        case 7: return conv_instance<NJ, 7, WL, U, TAIL>();
        case 8: return conv_instance<NJ, 8, WL, U, TAIL>();
    }
    return nullptr;
}

template <bool WL, int U, bool TAIL> ConvFn pick_tail_nj(int nj, int nv)
{
    switch (nj) {
        case 1: return pick_tail_nv<1, WL, U, TAIL>(nv);
        case 2: return pick_tail_nv<2, WL, U, TAIL>(nv);
        case 3: return pick_tail_nv<3, WL, U, TAIL>(nv);
        case 4: return pick_tail_nv<4, WL, U, TAIL>(nv);
        case 5: return pick_tail_nv<5, WL, U, TAIL>(nv);
        case 6: return pick_tail_nv<6, WL, U, TAIL>(nv);
        case 7: return pick_tail_nv<7, WL, U, TAIL>(nv);
        case 8: return pick_tail_nv<8, WL, U, TAIL>(nv);
    }
    return nullptr;
}

template <int U, bool TAIL> ConvFn pick_tail_kernel(int nj, int nv, bool wl)
{
    return wl ? pick_tail_nj<true, U, TAIL>(nj, nv) : pick_tail_nj<false, U, TAIL>(nj, nv);
}

}  // namespace conv

// One definition per translation unit direct_mfma_tail_u<U>.hip (with the 8-map block) and
// direct_mfma_plain_u<U>.hip (without).
conv::ConvFn conv_tail_kernel_u1(int nj, int nv, bool wl);
conv::ConvFn conv_tail_kernel_u2(int nj, int nv, bool wl);
conv::ConvFn conv_tail_kernel_u3(int nj, int nv, bool wl);
conv::ConvFn conv_tail_kernel_u4(int nj, int nv, bool wl);
conv::ConvFn conv_tail_kernel_u5(int nj, int nv, bool wl);
conv::ConvFn conv_tail_kernel_u7(int nj, int nv, bool wl);
conv::ConvFn conv_tail_kernel_u11(int nj, int nv, bool wl);
conv::ConvFn conv_plain_kernel_u1(int nj, int nv, bool wl);
conv::ConvFn conv_plain_kernel_u2(int nj, int nv, bool wl);
conv::ConvFn conv_plain_kernel_u3(int nj, int nv, bool wl);
conv::ConvFn conv_plain_kernel_u4(int nj, int nv, bool wl);
conv::ConvFn conv_plain_kernel_u5(int nj, int nv, bool wl);
conv::ConvFn conv_plain_kernel_u7(int nj, int nv, bool wl);
conv::ConvFn conv_plain_kernel_u11(int nj, int nv, bool wl);

}  // namespace znn
