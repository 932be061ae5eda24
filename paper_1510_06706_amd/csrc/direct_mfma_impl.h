// Kernel of the direct method on the fp32 matrix cores (forward and backward pass), shared
// by the translation units that instantiate it for one x-tap group width each.
//
//   D[m][n] += A[m][k] * B[k][n]      v_mfma_f32_16x16x4_f32
//     m : 16 output maps            (A = packed kernel weights, one coalesced load)
//     n : 16 output voxels          (B = input voxels read from an LDS halo tile)
//     k : 4 input maps at one kernel tap
//
// A workgroup of four waves owns a box of output voxels for up to 128 output maps; per
// chunk of four input maps it stages the input halo box in LDS once and walks all taps
// over it.
//
// What the tap loop is built around: on this hardware a scalar instruction or an LDS /
// global load issued between two MFMAs is nearly free, but every ordinary vector-ALU
// instruction costs the matrix pipeline several cycles (most when it sits alone between
// two MFMAs).  So the loop keeps vector arithmetic out of the per-tap path:
//   * taps are walked in groups of U neighbours along x; the B addresses of a group are
//     one base per voxel tile (NV vector additions per group, issued back to back) plus
//     immediate offsets per tap;
//   * tap offsets, weight pointers and loop counters are stepped in scalar registers;
//   * two operand register sets take turns (no copies); the loads of tap t+1 are issued
//     before the MFMAs of tap t.
// U = 1 is the general form (any kernel width, any sparsity); U > 1 needs taps one voxel
// apart along x and a kernel width that is a multiple of U.
#pragma once

#include "znn_internal.h"

namespace znn {
namespace conv {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) const void* global_cptr;
typedef __attribute__((address_space(3))) void* lds_ptr;
// Operand addresses in LDS are kept as 32-bit LDS pointers that already include the buffer's base: an
// operand read is then one ds_read with an immediate offset, and a tap group costs one vector addition
// per operand (an index added to the base at every use costs a second one).
typedef __attribute__((address_space(3))) const float* lds_floatp;

struct ConvTile {
    const float* src;   // K-side images [fK][sz][sy][sx]
    const float* wp;    // packed weights [jgroup][chunk][tap][NJ][64]
    float* dst;         // M-side images [fM][dz][dy][dx]
    int fK, fM;
    int sz, sy, sx;     // source extents
    int pz, py, px;     // zeros virtually in front of the source on each axis
    int dz, dy, dx;     // output extents
    int kz, ky, kx;
    int spz, spy, spx;  // sparsity: taps are this many voxels apart
    int Tz, Ty, Tx;     // output voxels per workgroup
    int HZ, HY, HX, MS; // halo box and LDS stride between the four staged maps
    int cz, cy, cx;     // workgroups per axis
    int nchunk;         // ceil(fK / 4)
    int cps;            // chunks per workgroup along gridDim.z (all of them unless the input maps are split)
    int dbuf;           // 1: two halo buffers take turns (next chunk in flight during the taps), 0: one buffer
    float* partial;     // [splits][fM][dz][dy][dx] partial sums when the input maps are split, else unused
    FastDiv dHX, dHY, dHZ;  // the halo loader takes its flat index apart without integer division
};

using ConvFn = void (*)(ConvTile);

// Walk over the tap groups of a chunk in (a, b, c-group) order, all in scalar registers.
// `o` is the halo offset of the group's lowest-address tap (its last one).
template <int U>
struct GroupWalk {
    int o, gc, gb;
    __device__ __forceinline__ void start(const ConvTile& P)
    {
        o = ((P.kz - 1) * P.spz * P.HY + (P.ky - 1) * P.spy) * P.HX + (P.kx - U) * P.spx;
        gc = 0; gb = 0;
    }
    __device__ __forceinline__ int step(const ConvTile& P, int groups_per_row)
    {
        int d = -U * P.spx;
        if (++gc == groups_per_row) {
            gc = 0;
            d += P.kx * P.spx - P.spy * P.HX;
            if (++gb == P.ky) { gb = 0; d += (P.ky * P.spy - P.spz * P.HY) * P.HX; }
        }
        return d;
    }
};

// One tap: the MFMAs of the current operand set, one row of map tiles at a time, with the
// B loads of the next tap dealt over the rows.  The fences keep the order written here: loads
// of the next tap go out while this tap's MFMAs run, and no vector arithmetic sits between
// MFMAs (the scheduler would otherwise put every load right in front of its first use).
template <int NJ, int NV>
__device__ __forceinline__ void tap_mfmas(floatx4 (&acc)[NJ][NV], const float (&a)[NJ], const float (&b)[NV],
                                          float (&bn)[NV], const lds_floatp (&vb)[NV], int imm)
{
#pragma unroll
    for (int jt = 0; jt < NJ; ++jt) {
#pragma unroll
        for (int nv = 0; nv < NV; ++nv) acc[jt][nv] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[jt], b[nv], acc[jt][nv], 0, 0, 0);
#pragma unroll
        for (int nv = jt * NV / NJ; nv < (jt + 1) * NV / NJ; ++nv) bn[nv] = vb[nv][imm];
        __builtin_amdgcn_sched_barrier(0);
    }
}

// The U taps of one group.  PAR: which operand set holds the group's first tap.  On entry
// that set is loaded (or in flight); on exit the other-parity set of the next group's first
// tap is in flight and vb / wg point at the next group.
//   vb[nv] : LDS address of the group's lowest-address tap for voxel tile nv (VGPR)
//   wg     : the group's packed weights (uniform pointer), wlo: the same as an LDS index when WL
template <int NJ, int NV, bool WL, int U, int PAR>
__device__ __forceinline__ void group_step(floatx4 (&acc)[NJ][NV], float (&a0)[NJ], float (&b0)[NV], float (&a1)[NJ],
                                           float (&b1)[NV], lds_floatp (&vb)[NV], const lds_floatp (&voff)[NV],
                                           const float*& wg, const float* wl, int& wlo, int lane, int o_next,
                                           bool advance)
{
#pragma unroll
    for (int u = 0; u < U; ++u) {
        float (&ac)[NJ] = ((PAR + u) & 1) ? a1 : a0;
        float (&bc)[NV] = ((PAR + u) & 1) ? b1 : b0;
        float (&an)[NJ] = ((PAR + u) & 1) ? a0 : a1;
        float (&bn)[NV] = ((PAR + u) & 1) ? b0 : b1;
        if (u + 1 < U) {
            // next tap of the same group: immediate offsets only
#pragma unroll
            for (int jt = 0; jt < NJ; ++jt)
                an[jt] = WL ? wl[wlo + ((u + 1) * NJ + jt) * 64] : wg[((u + 1) * NJ + jt) * 64 + lane];
            __builtin_amdgcn_sched_barrier(0);
            tap_mfmas<NJ, NV>(acc, ac, bc, bn, vb, U - 2 - u);
        } else {
            // first tap of the next group: new bases (the only vector arithmetic of the group)
            if (advance) {
                wg += U * NJ * 64;
                if (WL) wlo += U * NJ * 64;
            }
#pragma unroll
            for (int nv = 0; nv < NV; ++nv) vb[nv] = voff[nv] + o_next;
#pragma unroll
            for (int jt = 0; jt < NJ; ++jt) an[jt] = WL ? wl[wlo + jt * 64] : wg[jt * 64 + lane];
            __builtin_amdgcn_sched_barrier(0);
            tap_mfmas<NJ, NV>(acc, ac, bc, bn, vb, U - 1);
        }
    }
}

// WL: the packed weights of the current 4-map chunk are copied to LDS once per chunk and
// the A operands come from there.  Small kernels (few taps) go with small output boxes and
// few waves per SIMD, where a global load per tap would leave its whole latency exposed.
template <int NJ, int NV, bool WL, int U>
__global__ void __launch_bounds__(256, 2) k_conv_mfma(ConvTile P)
{
    extern __shared__ float lds[];
    const int taps = P.kz * P.ky * P.kx;
    // LDS: one or two halo buffers [4][MS] (two take turns when they fit), the table of the halo
    // loader [MSP], the chunk's weights [taps][NJ][64] when WL
    const int MSP = (P.MS + 255) & ~255;
    const int nbuf = P.dbuf ? 2 : 1;
    int* tab = reinterpret_cast<int*>(lds + nbuf * 4 * P.MS);
    float* wl = lds + nbuf * 4 * P.MS + MSP;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar
    const int col = lane & 15, grp = lane >> 4;

    int b = blockIdx.x;
    const int bxi = b % P.cx; b /= P.cx;
    const int byi = b % P.cy;
    const int bzi = b / P.cy;
    const int jg = blockIdx.y;
    const int z0 = bzi * P.Tz, y0 = byi * P.Ty, x0 = bxi * P.Tx;
    const int Ttot = P.Tz * P.Ty * P.Tx;

    lds_floatp voff[NV];
#pragma unroll
    for (int nv = 0; nv < NV; ++nv) {
        int t = (wave * NV + nv) * 16 + col;
        if (t >= Ttot) t = 0;
        const int tx = t % P.Tx, ty = (t / P.Tx) % P.Ty, tz = t / (P.Tx * P.Ty);
        voff[nv] = (lds_floatp)lds + (grp * P.MS + (tz * P.HY + ty) * P.HX + tx);
    }

    floatx4 acc[NJ][NV];
#pragma unroll
    for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
        for (int nv = 0; nv < NV; ++nv) acc[jt][nv] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int hvol = P.HZ * P.HY * P.HX;
    const long splane = (long)P.sy * P.sx;
    // this workgroup's share of the input-map chunks (all of them unless gridDim.z > 1)
    const int ic0 = blockIdx.z * P.cps, ic1 = min(P.nchunk, ic0 + P.cps);
    const float* wq = P.wp + ((long)jg * P.nchunk + ic0) * taps * NJ * 64;      // uniform
    const int groups_per_row = P.kx / U;
    const int ngroups = P.kz * P.ky * groups_per_row;

    // Halo loader.  Which voxel of a source map lands in which LDS word is the same for every
    // chunk, so it is worked out once: tab[r] = byte offset inside a map for word r of a map's
    // halo box, or -1 for words outside the image (zero padding) and behind the box.  Per chunk
    // a lane then needs no arithmetic: the map base is wave-uniform, the offset comes from the
    // table, and the data goes from global memory straight into LDS (no registers), so the
    // next chunk's box is fetched while this chunk's taps run.  Words with tab < 0 are zeroed
    // once and never written again.
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

    const long svol = (long)P.sz * splane;
    auto issue_chunk = [&](int ic, float* buf) {
        const int nvalid = min(4, P.fK - ic * 4);
        const char* cb = reinterpret_cast<const char*>(P.src + (long)ic * 4 * svol);    // uniform
        if (nvalid < 4)     // last chunk of a fan-in that is no multiple of four: the missing maps read as zero
            for (int q = nvalid * P.MS + threadIdx.x; q < 4 * P.MS; q += 256) buf[q] = 0.f;
        for (int r0 = 0; r0 < P.MS; r0 += 1024) {
            int tv[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) tv[j] = r0 + j * 256 < MSP ? tab[r0 + j * 256 + threadIdx.x] : -1;
            for (int m = 0; m < nvalid; ++m) {
                const char* mb = cb + (long)m * svol * 4;       // uniform
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int q0 = r0 + j * 256 + wave * 64;    // uniform
                    if (q0 < P.MS && tv[j] >= 0)
                        __builtin_amdgcn_global_load_lds((global_cptr)(mb + (unsigned)tv[j]), (lds_ptr)(buf + m * P.MS + q0), 4, 0, 0);
                }
            }
        }
    };

    if (P.dbuf && ic0 < ic1) issue_chunk(ic0, lds);
    for (int ic = ic0; ic < ic1; ++ic) {
        const int cur = P.dbuf ? (ic - ic0) & 1 : 0;
        if (!P.dbuf) {
            __syncthreads();                // everyone is done reading the previous chunk
            issue_chunk(ic, lds);
        }
        __builtin_amdgcn_s_waitcnt(0);      // this wave's share of the box has landed
        __syncthreads();                    // everyone's has, and nobody still reads the other buffer
        if (WL) {
            const floatx4* src4 = reinterpret_cast<const floatx4*>(wq);
            floatx4* dst4 = reinterpret_cast<floatx4*>(wl);
            for (int t = threadIdx.x; t < taps * NJ * 16; t += 256) dst4[t] = src4[t];
            __syncthreads();
        }
        if (P.dbuf && ic + 1 < ic1) issue_chunk(ic + 1, lds + (cur ^ 1) * 4 * P.MS);
        float a0[NJ], b0[NV], a1[NJ], b1[NV];
        lds_floatp vb[NV];
        GroupWalk<U> walk;
        walk.start(P);
        walk.o += cur * 4 * P.MS;           // the buffer's offset rides in the scalar tap offset
        const float* wg = wq;
        int wlo = lane;
#pragma unroll
        for (int nv = 0; nv < NV; ++nv) vb[nv] = voff[nv] + walk.o;
#pragma unroll
        for (int jt = 0; jt < NJ; ++jt) a0[jt] = WL ? wl[wlo + jt * 64] : wg[jt * 64 + lane];
#pragma unroll
        for (int nv = 0; nv < NV; ++nv) b0[nv] = vb[nv][U - 1];

        // groups are taken two at a time so that the operand-set parity at the top of the
        // loop body is a compile-time constant for odd U as well
        int g = 0;
        for (; g + 2 <= ngroups; g += 2) {
            walk.o += walk.step(P, groups_per_row);
            group_step<NJ, NV, WL, U, 0>(acc, a0, b0, a1, b1, vb, voff, wg, wl, wlo, lane, walk.o, true);
            const bool more = g + 2 < ngroups;
            walk.o += more ? walk.step(P, groups_per_row) : 0;
            group_step<NJ, NV, WL, U, (U & 1)>(acc, a0, b0, a1, b1, vb, voff, wg, wl, wlo, lane, walk.o, more);
            asm volatile("" ::: "memory");      // requests do not sink into the next iteration
        }
        if (g < ngroups)        // odd number of groups: the last one (its prefetch re-reads itself)
            group_step<NJ, NV, WL, U, 0>(acc, a0, b0, a1, b1, vb, voff, wg, wl, wlo, lane, walk.o, false);
        wq += (long)taps * NJ * 64;
    }

    // D[m][n]: lane holds rows m = 4*(lane/16) + r, column n = lane%16
    const long dplane = (long)P.dy * P.dx;
    float* out = gridDim.z > 1 ? P.partial + (long)blockIdx.z * P.fM * P.dz * dplane : P.dst;
#pragma unroll
    for (int nv = 0; nv < NV; ++nv) {
        const int t = (wave * NV + nv) * 16 + col;
        if (t >= Ttot) continue;
        const int tx = t % P.Tx, ty = (t / P.Tx) % P.Ty, tz = t / (P.Tx * P.Ty);
        const int z = z0 + tz, y = y0 + ty, x = x0 + tx;
        if (z >= P.dz || y >= P.dy || x >= P.dx) continue;
        const long vox = z * dplane + (long)y * P.dx + x;
#pragma unroll
        for (int jt = 0; jt < NJ; ++jt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int j = (jg * NJ + jt) * 16 + grp * 4 + r;
                if (j < P.fM) out[(long)j * P.dz * dplane + vox] = acc[jt][nv][r];
            }
    }
}

template <int NJ, bool WL, int U> ConvFn pick_nv(int nv)
{
    switch (nv) {
        case 2: return k_conv_mfma<NJ, 2, WL, U>;
        case 4: return k_conv_mfma<NJ, 4, WL, U>;
        case 5: if (NJ * 5 <= 40) return k_conv_mfma<NJ, (NJ * 5 <= 40 ? 5 : 2), WL, U>; break;
        case 6: if (NJ * 6 <= 40) return k_conv_mfma<NJ, (NJ * 6 <= 40 ? 6 : 2), WL, U>; break;
        case 7: if (NJ * 7 <= 40) return k_conv_mfma<NJ, (NJ * 7 <= 40 ? 7 : 2), WL, U>; break;
        case 8: if (NJ * 8 <= 40) return k_conv_mfma<NJ, (NJ * 8 <= 40 ? 8 : 2), WL, U>; break;
    }
    return nullptr;
}

template <bool WL, int U> ConvFn pick_nj(int nj, int nv)
{
    switch (nj) {
        case 1: return pick_nv<1, WL, U>(nv);
        case 2: return pick_nv<2, WL, U>(nv);
        case 3: return pick_nv<3, WL, U>(nv);
        case 4: return pick_nv<4, WL, U>(nv);
        case 5: return pick_nv<5, WL, U>(nv);
        case 6: return pick_nv<6, WL, U>(nv);
        case 7: return pick_nv<7, WL, U>(nv);
        case 8: return pick_nv<8, WL, U>(nv);
    }
    return nullptr;
}

template <int U> ConvFn pick_kernel(int nj, int nv, bool wl)
{
    return wl ? pick_nj<true, U>(nj, nv) : pick_nj<false, U>(nj, nv);
}

}  // namespace conv

// One definition per translation unit direct_mfma_u<U>.hip.
conv::ConvFn conv_kernel_u1(int nj, int nv, bool wl);
conv::ConvFn conv_kernel_u2(int nj, int nv, bool wl);
conv::ConvFn conv_kernel_u3(int nj, int nv, bool wl);
conv::ConvFn conv_kernel_u4(int nj, int nv, bool wl);
conv::ConvFn conv_kernel_u5(int nj, int nv, bool wl);
conv::ConvFn conv_kernel_u7(int nj, int nv, bool wl);
conv::ConvFn conv_kernel_u11(int nj, int nv, bool wl);

}  // namespace znn
