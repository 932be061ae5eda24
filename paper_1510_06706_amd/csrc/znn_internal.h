// Internal declarations shared by the host-side API and the kernel launchers.
// Nothing in here is part of the public boundary (that is include/znn.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "znn.h"

namespace znn {

// ---------------------------------------------------------------- errors
void set_error(const char* fmt, ...);
int  fail(int code, const char* fmt, ...);
// Checks hipGetLastError() after a launch; returns ZNN_OK or ZNN_EHIP.
int  check_launch(const char* what);

// ---------------------------------------------------------------- kernel-level tracing
// While tracing is on, every launch is bracketed by two HIP events on its stream.
struct TraceScope {
    TraceScope(const char* name, hipStream_t s);
    ~TraceScope();
    int slot;
    hipStream_t stream;
};
#define ZNN_LAUNCH(name, stream, kern, grid, block, lds, ...)                 \
    do {                                                                      \
        znn::TraceScope _ts(name, stream);                                    \
        hipLaunchKernelGGL(kern, grid, block, lds, stream, __VA_ARGS__);      \
    } while (0)

// ---------------------------------------------------------------- geometry
struct Geom {
    int f, fo;            // fan-in, fan-out
    int nz, ny, nx;       // image extents n
    int kz, ky, kx;       // kernel extents k
    int spz, spy, spx;    // sparsity s: neighbouring taps are s voxels apart (Section 2)
    int oz, oy, ox;       // n' = n - s (k - 1)
    int Nz, Ny, Nx, Nxh;  // FFT extents and N_x/2+1
    __host__ __device__ long nvol() const { return (long)nz * ny * nx; }
    __host__ __device__ long kvol() const { return (long)kz * ky * kx; }
    __host__ __device__ long ovol() const { return (long)oz * oy * ox; }
    __host__ __device__ long svol() const { return (long)Nz * Ny * Nxh; }   // complex elements per spectrum
};

inline size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

// Smallest 2^a 3^b 5^c >= n.
int  next_fft_extent(int n);
// Largest FFT extent the LDS-resident passes accept.
constexpr int kMaxFftExtent = 1024;

// Division of small unsigned numbers by a launch constant without a hardware divide:
// q = (n * M) >> 32 with M = floor(2^32 / d) + 1 is exact while n * d < 2^32.
struct FastDiv {
    unsigned d, M;
};
inline FastDiv make_fastdiv(unsigned d)
{
    FastDiv f;
    f.d = d;
    f.M = d <= 1 ? 0u : (unsigned)(((1ull << 32) / d) + 1ull);
    return f;
}
__device__ __forceinline__ unsigned fdiv(unsigned n, FastDiv f)
{
    return f.d <= 1 ? n : __umulhi(n, f.M);
}

// Tuning aids.  The environment is read exactly once, the first time anything asks (plan
// creation at the latest), and never on a launch path; none of them changes a data layout.
struct Tuning {
    bool log;                   // ZNN_LOG: print launch configurations to stderr
    bool conv_u1;               // ZNN_CONV_U1: walk the taps of the direct convolution one at a time
    bool conv_no_wl;            // ZNN_CONV_NO_WL: never stage a chunk's weights in LDS
    bool conv_no_split;         // ZNN_CONV_NO_SPLIT: never split the input maps over workgroups
    bool conv_no_tail;          // ZNN_CONV_NO_TAIL: pad the last maps to a 16-row tile instead of an 8-map block
    int  conv_tile[4];          // ZNN_CONV_TILE="NV,Tz,Ty,Tx": pin the output box (0 = not pinned)
    int  wgrad_halves;          // ZNN_WGRAD_HALVES: 1 = four waves, 2 = eight waves per workgroup
    int  wgrad_maxnj;           // ZNN_WGRAD_MAXNJ: most 16-map tiles per workgroup
    int  wgrad_own_waves;       // ZNN_WGRAD_OWN_WAVES: 4 or 8 waves per workgroup in that layout
    int  wgrad_own_columns_from; // ZNN_WGRAD_OWN_COLUMNS_FROM: column tiles from which every wave owns columns
    int  wgrad_stride_mod;      // ZNN_WGRAD_STRIDE_MOD: residue modulo 32 of the LDS map stride
    bool wgrad_slow_loader;     // ZNN_WGRAD_SLOW_LOADER: general tile loader everywhere
    int  fft_mac_z0;            // ZNN_FFT_MAC_Z0: frequencies per thread of the folded multiply-accumulate / 4
    bool fft_mac_valu;          // ZNN_FFT_MAC_VALU: folded multiply-accumulate on the vector ALUs only
    bool fft_wgrad_plain;       // ZNN_FFT_WGRAD_PLAIN: per-z pruned DFT instead of the radix-4 grouped one
    bool fft_no_fused_xy;       // ZNN_FFT_NO_FUSED_XY: separate x and y passes even where one launch can take both
    bool fft_no_two_level;      // ZNN_FFT_NO_TWO_LEVEL: 256-point strided passes through the LDS radix passes
    bool fft_no_mac_inverse;    // ZNN_FFT_NO_MAC_INVERSE: inverse transform along z as a pass of its own, never inside the multiply-accumulate
    bool fft_no_taps_pass;      // ZNN_FFT_NO_TAPS_PASS: kernels take the general fused x/y pass
    int  fft_lds_kb;            // ZNN_FFT_LDS_KB: LDS per workgroup of the LDS passes (pencils per workgroup follow); 0 = per pass kind
    bool fft_lds_passes;        // ZNN_FFT_LDS_PASSES: LDS passes instead of register passes
};
const Tuning& tuning();
inline bool log_enabled() { return tuning().log; }

// ---------------------------------------------------------------- direct method
int direct_fwd(const Geom& g, const float* in, const float* w, float* out, void* ws, hipStream_t s);
int direct_bwd(const Geom& g, const float* gout, const float* w, float* gin, void* ws, hipStream_t s);
int direct_wgrad(const Geom& g, const float* in, const float* gout, float* gw, void* ws, hipStream_t s);
size_t direct_workspace_bytes(const Geom& g, int pass);

// ---------------------------------------------------------------- FFT method
// Layout of a layer's kernel spectra, fixed when its plan is created (or by
// znn_plan_set_spectra_layout) and carried by the plan from then on, so that the size query,
// the kernel transform and every multiply-accumulate read the same decision.
//   on = false : full spectra [f'][f][N_z][N_y][N_x/2+1] (Section 4, memoized kernel transforms)
//   on = true  : half spectra [f'][f][taps][P], transformed along the fast axes only; the sum
//                over the `taps` planes of the slowest axis (extent N) is taken inside the
//                multiply-accumulate, 4*z0 frequencies per thread
struct Fold { bool on; int N, taps, P, z0; };
Fold fold_full();
// The library's own choice: half spectra where the folded multiply-accumulate applies and the
// layer has enough frequencies to fill the chip, else full spectra.
Fold fold_default(const Geom& g);
// Half spectra whenever the folded multiply-accumulate can take the layer at all (on = false if not).
Fold fold_forced(const Geom& g);

struct FftWorkspace {
    size_t total;
    size_t off_a, off_b;        // spectra of the two node sets of the pass
    size_t off_w;               // kernel spectra (when not resident)
    size_t off_t1, off_t2;      // partially inverted pair volumes (kernel gradient)
};
FftWorkspace fft_workspace(const Geom& g, const Fold& F, int pass, bool resident);
size_t fft_spectra_bytes(const Geom& g, const Fold& F);
int fft_kernel_spectra(const Geom& g, const Fold& F, const float* w, float2* What, hipStream_t s);
int fft_fwd(const Geom& g, const Fold& F, const float* in, const float* w, const float2* resident, float* out,
            void* ws, float2* memo_in, hipStream_t s);
int fft_bwd(const Geom& g, const Fold& F, const float* gout, const float* w, const float2* resident, float* gin,
            void* ws, float2* memo_gout, hipStream_t s);
int fft_wgrad(const Geom& g, const float* in, const float* gout, float* gw, void* ws, hipStream_t s);
int fft_wgrad_from_spectra(const Geom& g, const float2* Ihat, const float2* Ghat, float* gw, void* ws,
                           hipStream_t s);

// Multiply-accumulate with the kernel transform's last axis folded in (fft_mac.hip):
// Wh holds half spectra [pair][tap][P]; X, Y are node spectra [node][N][P].
constexpr int kMaxFoldedTaps = 16;
// z0 = 4, 2 or 1: frequencies per thread along the folded axis are 4 * z0; a thread serves
// fft_mac_group(z0) result nodes.
constexpr int fft_mac_group(int z0) { return z0 == 1 ? 8 : 4; }
int fft_mac_fused(bool backward, int taps, int z0, int f, int fo, int N, int P, const float2* Wh,
                  const float2* X, float2* Y, hipStream_t s);

// The same with the rebuild of the kernel spectrum on the matrix cores (fft_mac_mfma.hip); takes
// extents divisible by 32.
bool fft_mac_mfma_supported(int taps, int N, int P);
bool fft_mac_mfma_can_invert(int taps, int N, int P, int nout);
int fft_mac_mfma(bool backward, int taps, int f, int fo, int N, int P, const float2* Wh, const float2* X,
                 float2* Y, int zinv_o0, int zinv_no, hipStream_t s);
// (zinv_no > 0: the rows [zinv_o0, zinv_o0 + zinv_no) of Y receive the inverse transform of the sums along
// the folded axis instead of the sums; only where fft_mac_mfma_can_invert says so)

// Strided-axis FFT pass with one pencil per thread, whole pencil in registers (fft_reg.hip).
// Pencil (oa, ob, l), l < L, has its element e at in + oa*in_sa + ob*in_sb + l + e*stride;
// elements outside [i0, i0+ni) are taken as zero, only [o0, o0+no) are written.
struct RegAxis {
    const float2* in; float2* out;
    int N, i0, ni, o0, no;
    long stride;
    int L, Oa, Ob;
    long in_sa, in_sb, out_sa, out_sb;
    FastDiv fL;
};
bool fft_axis_reg_supported(int N);
int  fft_axis_reg(RegAxis P, int dir, hipStream_t s);

// Strided-axis FFT passes of lengths N = N1 * N2 above the register limit, N1, N2 <= 16, in two levels with
// the samples in registers at both (fft_two_level.hip).  Pencil (oa, ob, oc, l), l < L, has element e at
// in + oa*in_sa + ob*in_sb + oc*in_sc + l + e*in_stride; elements outside [i0, i0+ni) are taken as zero,
// only [o0, o0+no) are written.
struct TwoLevelAxis {
    const float2* in; float2* out;
    int N, i0, ni, o0, no;
    long in_stride, out_stride;
    int L, Oa, Ob, Oc;
    long in_sa, in_sb, in_sc, out_sa, out_sb, out_sc;
    int chunks;                     // chunks of 16 neighbouring pencils per run of L (filled by the launcher)
    FastDiv fchunks, foc, fob;
};
bool fft_axis_two_level_supported(int N);
int  fft_axis_two_level(TwoLevelAxis P, int dir, hipStream_t s);

// x-axis passes with one row per thread and the row's transform in registers (fft_x_reg*.hip).
// r2c: rows of `sx` real samples (contiguous, `rows` = maps * sz * sy of them) land zero-extended from
// offset ox in lines of N = 2 (Nxh - 1); row (map, z, y) goes to spectrum row (map, z*tz + oz, y*ty + oy).
struct XRegR2C {
    const float* src; float2* dst;
    long rows;
    int sz, sy, sx;
    int Nz, Ny, Nxh;
    int oz, oy, ox;
    int tz, ty;
    FastDiv fsy, fsz;
};
// c2r: spectrum rows (map, z + cz, y + cy), z < dz, y < dy, become contiguous rows of the dx real
// samples from offset cx, times `scale`.
struct XRegC2R {
    const float2* src; float* dst;
    long rows;
    int cz, cy, cx;
    int dz, dy, dx;
    int Nz, Ny, Nxh;
    float scale;
    FastDiv fdy, fdz;
};
// x and y passes in one launch for volumes with equal x and y transform lengths N (fft_xy_reg*.hip):
// a (map, z) plane per workgroup.  forward: planes = maps * sz real planes of sy rows x sx samples, placed
// at (z * tz + oz, oy, ox); inverse: planes = maps * dz spectrum planes z + cz, cropped to rows [cy, cy+dy)
// and samples [cx, cx+dx), times `scale`.
struct XYFwd {
    const float* src; float2* dst;
    long planes;
    int sz, sy, sx;
    int Nz, oz, oy, ox, tz;
};
struct XYInv {
    const float2* src; float* dst;
    long planes;
    int dz, dy, dx;
    int Nz, cz, cy, cx;
    float scale;
};
bool fft_xy_reg_supported(int N);
int  fft_xy_fwd_reg(const XYFwd& P, int N, hipStream_t s);
int  fft_xy_inv_reg(const XYInv& P, int N, hipStream_t s);
bool fft_x_reg_supported(int N);
int  fft_x_r2c_reg(const XRegR2C& P, int N, hipStream_t s);
int  fft_x_c2r_reg(const XRegC2R& P, int N, hipStream_t s);

// ---------------------------------------------------------------- fill (autotuner)
int fill_pattern(float* p, long count, float scale, hipStream_t s);

}  // namespace znn

struct znn_plan {
    znn_conv_desc desc;
    znn::Geom g;
    int mode;                    // ZNN_DIRECT or ZNN_FFT
    znn::Fold fold;              // layout of this layer's kernel spectra (FFT method)
    const float2* resident;      // kernel spectra held by the caller, or nullptr
    float2* memo;                // caller's buffer for memoized node spectra, or nullptr
    bool memo_has_in, memo_has_gout;
};
