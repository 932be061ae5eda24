// Direct method on the fp32 matrix cores (forward and backward pass): what the kernel in
// direct_mfma_tail_impl.h shares with the host side (tile description, tap walk), and how the kernel is built.
//
//   D[m][n] += A[m][k] * B[k][n]      v_mfma_f32_16x16x4_f32
//     m : 16 output maps            (A = packed kernel weights, one coalesced load)
//     n : 16 output voxels          (B = input voxels read from an LDS halo tile)
//     k : 4 input maps at one kernel tap
//   (the last 1..8 maps of a count that is no multiple of 16 run on v_mfma_f32_4x4x1_16B_f32 instead of a
//   padded tile: direct_mfma_tail_impl.h)
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
    const float* wp;    // packed weights [jgroup][chunk][tap][NJ][64] (+ [8][4] per tap with an 8-map block)
    float* dst;         // M-side images [fM][dz][dy][dx]
    int fK, fM;
    int sz, sy, sx;     // source extents
    int pz, py, px;     // zeros virtually in front of the source on each axis
    int dz, dy, dx;     // output extents
    int kz, ky, kx;
    int spz, spy, spx;  // sparsity: taps are this many voxels apart
    int Tz, Ty, Tx;     // output voxels per workgroup
    int HZ, HY, HX, MS; // halo box; MS = its voxels rounded up to 16 (a halo buffer holds 4 * MS words, maps interleaved)
    int cz, cy, cx;     // workgroups per axis
    int nchunk;         // ceil(fK / 4)
    int cps;            // chunks per workgroup along gridDim.z (all of them unless the input maps are split)
    int dbuf;           // 1: two halo buffers take turns (next chunk in flight during the taps), 0: one buffer
    float* partial;     // [splits][fM][dz][dy][dx] partial sums when the input maps are split, else unused
    FastDiv dHX, dHY, dHZ;  // the halo loader takes its flat index apart without integer division
};

using ConvFn = void (*)(ConvTile);

// Walk over the tap groups of a chunk in (a, b, c-group) order, all in scalar registers.
// `o` is the halo offset of the group's lowest-address tap (its last one).  Packed tap (a, b, c) meets the
// halo at tap offset (kz-1-a, ky-1-b, kx-1-c).  The walk covers `na` planes and `nb` rows of taps, the ones
// at halo offsets alpha_hi down and beta_hi down: a workgroup whose box lies at the border of a zero-extended
// source (backward pass) leaves out the planes and rows of taps that meet nothing but the padding.
template <int U>
struct GroupWalk {
    int o, gc, gb, nb, wrow;
    // wrow: packed weights (floats) of the tap rows a plane of the walk leaves out
    __device__ __forceinline__ void start(const ConvTile& P, int alpha_hi, int beta_hi, int rows, int skipped_row_floats)
    {
        o = (alpha_hi * P.spz * P.HY + beta_hi * P.spy) * P.HX + (P.kx - U) * P.spx;
        gc = 0; gb = 0; nb = rows; wrow = skipped_row_floats;
    }
    // step to the next group: returns the change of `o`; `wd` (floats to the next group's packed weights)
    // grows by the rows left out when the walk enters the next plane
    __device__ __forceinline__ int step(const ConvTile& P, int groups_per_row, int& wd)
    {
        int d = -U * P.spx;
        if (++gc == groups_per_row) {
            gc = 0;
            d += P.kx * P.spx - P.spy * P.HX;
            if (++gb == nb) { gb = 0; d += (nb * P.spy - P.spz * P.HY) * P.HX; wd += wrow; }
        }
        return d;
    }
};

// Range [lo, hi] of tap offsets t (in taps, `sp` voxels apart, t < k) along one axis for which the rows
// origin + i + t * sp - pad, i < n, of the source meet [0, extent); hi < lo: none.
__device__ __forceinline__ void live_taps(int origin, int n, int pad, int extent, int k, int sp, int& lo, int& hi)
{
    const int first = pad - origin - (n - 1), last = pad - origin + extent - 1;     // t * sp in [first, last]
    lo = first <= 0 ? 0 : (first + sp - 1) / sp;
    hi = last < 0 ? -1 : min(k - 1, last / sp);
}

}  // namespace conv

}  // namespace znn
