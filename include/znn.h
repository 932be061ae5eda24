/*
 * znn.h -- C ABI of the MI355X (gfx950) convolutional-layer library.
 *
 * The library computes the per-edge 3D convolutions of a ConvNet computation
 * graph in the sense of ZNN (arXiv 1510.06706, Section 2): a layer has f input
 * nodes and f' output nodes joined by f*f' convolution edges, and a node sums
 * the outputs of the edges that converge on it.  All three training passes are
 * provided (forward, backward, kernel gradient; Sections 2, 3.1, 3.2), each by
 * the direct method or by the FFT method (Section 4), together with the
 * sliding-window max-filter and its Jacobian and the per-layer choice between
 * the two methods.
 *
 * Conventions common to every entry point
 *   - All tensor pointers are DEVICE pointers to dense fp32 (or int32) arrays,
 *     row-major with x fastest:
 *        images   [map][z][y][x]
 *        kernels  [fan_out][fan_in][kz][ky][kx]
 *     2D is the special case z-extent 1.  Extents may differ per axis.
 *   - The caller owns every buffer.  Outputs are overwritten, inputs are never
 *     modified, inputs and outputs must not overlap.  Scratch memory comes from
 *     the caller's workspace `ws` (256-byte aligned, size from
 *     znn_plan_workspace_bytes); the compute entry points never allocate or
 *     free device memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Every entry point only enqueues work on `stream` and returns; it never
 *     synchronises with the host (znn_autotune is the one exception).
 *   - Return value: ZNN_OK or a negative error code; a description of the last
 *     error on the calling thread is available from znn_last_error().  Nothing
 *     throws or aborts across this boundary.  Argument validation happens on
 *     the host before anything is launched.
 */
#ifndef ZNN_H
#define ZNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ZNN_OK             0
#define ZNN_EINVAL       (-1)  /* null pointer, extent < 1, kernel or window larger than image */
#define ZNN_EUNSUPPORTED (-2)  /* index range beyond int32, FFT extent too large               */
#define ZNN_EWORKSPACE   (-3)  /* workspace (or spectra buffer) missing, misaligned or too small  */
#define ZNN_EHIP         (-4)  /* the HIP runtime reported an error; see znn_last_error()          */

typedef struct { int32_t z, y, x; } znn_vec3;

typedef enum { ZNN_DIRECT = 0, ZNN_FFT = 1, ZNN_AUTO = 2 } znn_mode;
typedef enum { ZNN_PASS_FWD = 0, ZNN_PASS_BWD = 1, ZNN_PASS_WGRAD = 2 } znn_pass;

/* One fully connected convolutional layer (Section 2; Table 2 uses the same f, f', n, k). */
typedef struct {
    int32_t  fan_in;      /* f  >= 1 : number of input nodes                                */
    int32_t  fan_out;     /* f' >= 1 : number of output nodes                               */
    znn_vec3 image;       /* n  : extents of every input image                              */
    znn_vec3 kernel;      /* k  : extents of every kernel, k_d >= 1, s_d (k_d - 1) + 1 <= n_d */
    znn_vec3 sparsity;    /* s  : s_d >= 1; neighbouring taps are s_d voxels apart (Section 2,
                             sparse convolution), outputs have extents n - s (k - 1);
                             {1,1,1} is the ordinary dense convolution                      */
    int32_t  mode;        /* znn_mode; ZNN_AUTO takes the autotuner's cached choice for this
                             descriptor, or a cost-model guess when nothing is cached       */
} znn_conv_desc;

typedef struct znn_plan znn_plan;   /* opaque host object: method, FFT extents, resident spectra */

/* Host only.  Validates the descriptor and fixes the method and the FFT extents
 * N_d (the smallest 2^a 3^b 5^c >= n_d per axis).  *plan is set on success only. */
int  znn_plan_create(const znn_conv_desc* desc, znn_plan** plan);
void znn_plan_destroy(znn_plan* plan);

/* Host only queries.  mode is ZNN_DIRECT or ZNN_FFT (never ZNN_AUTO). */
int  znn_plan_mode(const znn_plan* plan, int32_t* mode);
int  znn_plan_fft_extents(const znn_plan* plan, znn_vec3* N);
/* Bytes of workspace the given pass (znn_pass) needs with the plan's method and
 * its current state (resident kernel spectra make forward/backward smaller). */
int  znn_plan_workspace_bytes(const znn_plan* plan, int32_t pass, size_t* bytes);
/*
 * Layout of a layer's kernel spectra (complex fp32), a property of the plan (Section 4,
 * "FFT memoization"; Table 2, column "FFT-based (Memoized)").
 *   ZNN_SPECTRA_FULL    the transforms themselves, W^[f'][f][N_z][N_y][N_x/2+1]: what the
 *                       paper memoizes.  The multiply-accumulate streams them from HBM once
 *                       per pass and is bound by that stream (8 bytes per 8 FLOP).
 *   ZNN_SPECTRA_FOLDED  "half spectra" [f'][f][k_z][N_y][N_x/2+1] (2D: [f'][f][k_y][N_x/2+1]),
 *                       transformed along the fast axes only; the sum over the k_z planes of
 *                       the slowest axis is taken inside the multiply-accumulate.  N_z / k_z
 *                       times fewer bytes, arithmetic-bound.  Needs the slowest non-trivial
 *                       axis to have an FFT extent divisible by 4 and at most 16 taps one
 *                       voxel apart along it (ZNN_EUNSUPPORTED otherwise).
 *   ZNN_SPECTRA_AUTO    the library's choice: folded where it applies and the layer has
 *                       enough frequencies to fill the chip, else full.  This is what
 *                       znn_plan_create selects.
 * The choice is stored in the plan when it is created or set and read from there by the size
 * queries, the kernel transform and both multiply-accumulates.  znn_plan_set_spectra_layout
 * is host only, valid for FFT plans, and fails with ZNN_EINVAL while resident spectra are
 * attached (release them first): a buffer is only ever read in the layout it was written in.
 * Workspace and spectra sizes must be queried again after a change.
 * znn_plan_spectra_layout reports ZNN_SPECTRA_FULL or ZNN_SPECTRA_FOLDED, never AUTO.
 */
typedef enum { ZNN_SPECTRA_AUTO = 0, ZNN_SPECTRA_FULL = 1, ZNN_SPECTRA_FOLDED = 2 } znn_spectra_layout;
int  znn_plan_set_spectra_layout(znn_plan* plan, int32_t layout);
int  znn_plan_spectra_layout(const znn_plan* plan, int32_t* layout);
/* Bytes of the kernel spectra in the plan's layout. */
int  znn_plan_spectra_bytes(const znn_plan* plan, size_t* bytes);

/*
 * FFT method only: transform all f*f' kernels once and keep their spectra in
 * the caller's buffer `spectra` (device, 256-byte aligned, at least
 * znn_plan_spectra_bytes).  This is the kernel half of the FFT memoization of
 * Section 4.  Afterwards znn_conv3d_fwd / znn_conv3d_bwd on this plan ignore
 * their `w` argument (it may be NULL) and stream the resident spectra.  The
 * buffer stays owned by the caller and must outlive the plan or a later
 * znn_conv_release_kernels.  `ws` needs no more than the forward workspace.
 */
int  znn_conv_prepare_kernels(znn_plan* plan, const float* w, void* spectra, size_t spectra_bytes,
                              void* ws, size_t ws_bytes, void* stream);
int  znn_conv_release_kernels(znn_plan* plan);

/*
 * FFT method only: memoization of the node spectra (Section 4; Table 2, column
 * "FFT-based (Memoized)").  While a caller-owned buffer `memo` (device, 256-byte
 * aligned, at least znn_plan_memo_bytes) is attached, znn_conv3d_fwd leaves the
 * spectra of its input images there and znn_conv3d_bwd the spectra of its output
 * gradients; znn_conv3d_wgrad_memo then computes the kernel gradient of exactly
 * those two tensors without transforming them again (only the f*f' pruned inverse
 * transforms remain).  It fails with ZNN_EINVAL unless both passes have run on this
 * plan since the buffer was attached; each later forward / backward call replaces
 * its half.  memo = NULL detaches.  Results are bit-identical to znn_conv3d_wgrad.
 */
int  znn_plan_memo_bytes(const znn_plan* plan, size_t* bytes);
int  znn_conv_set_memo(znn_plan* plan, void* memo, size_t memo_bytes);
int  znn_conv3d_wgrad_memo(znn_plan* plan, float* gw, void* ws, size_t ws_bytes, void* stream);

/*
 * Forward pass (Section 2, "Convolution", and the node sum of the computation
 * graph): out[j] = sum_i valid_conv(in[i], w[j][i]), a true convolution (kernel
 * index runs against the image index), output extents n' = n - s (k - 1):
 *   out[j][x] = sum_i sum_a w[j][i][a] in[i][x + s (k - 1 - a)]   (per axis)
 * With sparsity s > 1 only every s-th voxel of the window enters the sum.
 *   in  [f][n]   w [f'][f][k]   ->   out [f'][n']
 */
int  znn_conv3d_fwd(znn_plan* plan, const float* in, const float* w, float* out,
                    void* ws, size_t ws_bytes, void* stream);

/*
 * znn_conv3d_fwd for callers that cannot allocate device memory and therefore have no
 * workspace to hand over: code running under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, results and error codes as
 * znn_conv3d_fwd (either method; `w` may be NULL with resident spectra), bit for bit the same
 * output, but the scratch comes from a device array of ZNN_STATIC_SCRATCH_BYTES built into the
 * library, of which every GPU the library runs on holds its own copy until the process ends.
 * The call allocates and frees nothing.  A layer whose forward pass needs more scratch than
 * that (znn_plan_workspace_bytes) is refused with ZNN_EWORKSPACE before anything is launched.
 * All calls on one GPU share the one array: calls that may overlap in time on the same GPU (two
 * streams, two threads) race and must be serialised by the caller; calls on one stream are safe.
 * The array's device address is looked up on the first call per device, with that device current.
 */
#define ZNN_STATIC_SCRATCH_BYTES (32u * 1024u * 1024u)
int  znn_conv3d_fwd_static(znn_plan* plan, const float* in, const float* w, float* out, void* stream);

/*
 * Backward pass (Section 3.1, "Convolution Jacobian"): full convolution of the
 * output gradients with the kernel reflected along all three axes, summed over
 * the outgoing edges of each input node.
 *   gout [f'][n']   w [f'][f][k]   ->   gin [f][n]
 */
int  znn_conv3d_bwd(znn_plan* plan, const float* gout, const float* w, float* gin,
                    void* ws, size_t ws_bytes, void* stream);

/*
 * Kernel gradient (Section 3.2, "Kernel update"): valid convolution of the
 * reflected forward image at the source node with the backward image at the
 * target node, kernel-sized.
 *   in [f][n]   gout [f'][n']   ->   gw [f'][f][k]
 */
int  znn_conv3d_wgrad(znn_plan* plan, const float* in, const float* gout, float* gw,
                      void* ws, size_t ws_bytes, void* stream);

/*
 * Max-filtering (Section 2): out[m][p] = max over the window p + [0, win) of
 * in[m]; extents n - win + 1.  idx[m][p] is the flat offset (z*n_y + y)*n_x + x
 * inside map m of the voxel that supplied the maximum; among equal values the
 * smallest offset wins (+0 and -0 are equal).  Inputs must not contain NaN.
 *   in [maps][n]  ->  out [maps][n-win+1] (fp32), idx [maps][n-win+1] (int32)
 */
int  znn_maxfilter3d_fwd(int32_t maps, znn_vec3 n, znn_vec3 win, const float* in,
                         float* out, int32_t* idx, void* stream);

/*
 * Max-filtering Jacobian (Section 3.1): gin is a zero image of the filter's
 * input extents n into which every gout[m][p] is accumulated at idx[m][p].
 * idx must come from znn_maxfilter3d_fwd with the same maps, n and win (every
 * recorded offset lies inside its own window); the sum for a voxel is taken in
 * ascending window order, so results are reproducible bit for bit.
 */
int  znn_maxfilter3d_bwd(int32_t maps, znn_vec3 n, znn_vec3 win, const float* gout,
                         const int32_t* idx, float* gin, void* stream);

/*
 * Max-filtering whose window taps lie `sparsity` voxels apart; extents
 * n - s (win - 1).  In a max-filtering ConvNet every filter multiplies the
 * sparsity of all later layers by its window (Section 2, last paragraphs and
 * the figure there); that includes later filters, which is what makes the net
 * reproduce a sliding-window max-pooling ConvNet voxel for voxel.  Same idx
 * convention, tie rule and reproducible summation order as the dense calls
 * above, which are these with sparsity {1,1,1}.
 */
int  znn_maxfilter3d_sparse_fwd(int32_t maps, znn_vec3 n, znn_vec3 win, znn_vec3 sparsity,
                                const float* in, float* out, int32_t* idx, void* stream);
int  znn_maxfilter3d_sparse_bwd(int32_t maps, znn_vec3 n, znn_vec3 win, znn_vec3 sparsity,
                                const float* gout, const int32_t* idx, float* gin, void* stream);

/*
 * Max-pooling (Section 2) and its Jacobian (Section 3.1).  The image is cut into
 * blocks of p voxels per axis; n must be divisible by p (ZNN_EINVAL otherwise).
 *   fwd: in [maps][n] -> out [maps][n/p] (block maxima), idx [maps][n/p] (flat offset
 *        inside the input map of the voxel that supplied each maximum; among equal
 *        values the smallest offset wins)
 *   bwd: gout [maps][n/p], idx -> gin [maps][n]: all voxels of a block are zero except
 *        the recorded one, which receives the block's gout.  Every gin voxel is written.
 */
int  znn_maxpool3d_fwd(int32_t maps, znn_vec3 n, znn_vec3 p, const float* in,
                       float* out, int32_t* idx, void* stream);
int  znn_maxpool3d_bwd(int32_t maps, znn_vec3 n, znn_vec3 p, const float* gout,
                       const int32_t* idx, float* gin, void* stream);

/*
 * Transfer-function edges and the update step that a training round needs
 * around the convolutions (Sections 2, 3.1, 3.2).  All are elementwise or
 * per-map reductions over images [maps][voxels].
 *   znn_transfer_fwd : y = max(x + bias[m], 0)             (half-wave rectification)
 *   znn_transfer_bwd : gx = gy * (y > 0 ? 1 : 0)           (y = forward output)
 *   znn_bias_grad    : gb[m] = sum of all voxels of g[m]   (fixed summation order)
 *   znn_square_loss_grad : g = out - target                (loss 1/2 sum (out-target)^2)
 *   znn_sgd_update   : p -= eta * g                        (Algorithm 3)
 * znn_transfer_fn_fwd / _bwd take the nonlinearity as an argument: the three the
 * paper names (Section 2, "Transfer function").  The backward edge multiplies gy by
 * the derivative written through the forward output y.  ZNN_EINVAL for other values.
 *   znn_cross_entropy_loss_grad : g = (out - target) / (out (1 - out)), the gradient of
 *       - sum target log out + (1 - target) log (1 - out); out must lie strictly
 *       inside (0, 1) (the partner of a logistic output layer).  The paper names the
 *       Euclidean loss and leaves the others open; this is the second one built.
 */
typedef enum znn_transfer_fn {
    ZNN_RECTIFY  = 0,   /* y = max(v, 0)              dy/dv = (y > 0)    */
    ZNN_LOGISTIC = 1,   /* y = 1 / (1 + exp(-v))      dy/dv = y (1 - y)  */
    ZNN_TANH     = 2    /* y = tanh(v)                dy/dv = 1 - y^2    */
} znn_transfer_fn;

int  znn_transfer_fwd(int32_t maps, int64_t voxels, const float* x, const float* bias, float* y, void* stream);
int  znn_transfer_bwd(int32_t maps, int64_t voxels, const float* gy, const float* y, float* gx, void* stream);
int  znn_bias_grad(int32_t maps, int64_t voxels, const float* g, float* gb, void* stream);
int  znn_transfer_fn_fwd(int32_t fn, int32_t maps, int64_t voxels, const float* x, const float* bias, float* y,
                         void* stream);
int  znn_transfer_fn_bwd(int32_t fn, int32_t maps, int64_t voxels, const float* gy, const float* y, float* gx,
                         void* stream);
int  znn_square_loss_grad(int64_t count, const float* out, const float* target, float* g, void* stream);
int  znn_cross_entropy_loss_grad(int64_t count, const float* out, const float* target, float* g, void* stream);
int  znn_sgd_update(int64_t count, float eta, const float* g, float* p, void* stream);

/*
 * Node sum of a general computation graph (Section 2: a node's image is the sum of the
 * outputs of the edges converging on it; Section 3.1: a node's backward image is the
 * sum over its outgoing edges): y += x, elementwise.  The convolution calls above sum
 * the edges of ONE fully connected bundle themselves; this adds the results of several
 * bundles (branches with different kernels or sparsity) that meet at one node.
 */
int  znn_accumulate(int64_t count, const float* x, float* y, void* stream);

/*
 * Layer-wise choice between the direct and the FFT method (Section 4): times
 * forward + backward + kernel gradient in both methods on the given shape
 * (2 warm-up rounds, 5 timed), stores the faster one in a process-wide cache
 * keyed by the descriptor (consulted by znn_plan_create for ZNN_AUTO) and
 * reports it.  ms[method][pass] receives the mean milliseconds.  The tensors
 * are carved from `ws` and filled with a fixed pattern; `ws` must hold
 * znn_autotune_workspace_bytes.  Synchronises `stream` with the host.
 */
int  znn_autotune_workspace_bytes(const znn_conv_desc* desc, size_t* bytes);
int  znn_autotune(const znn_conv_desc* desc, void* ws, size_t ws_bytes, void* stream,
                  int32_t* chosen_mode, float ms[2][3]);

/*
 * Whole-round choice under a memory budget (Section 4: memoizing the transforms
 * of images and kernels trades memory for a third fewer transforms, Table 2).
 * Three ways to run one training round of a layer are timed as a whole
 * (forward, then backward, then kernel gradient; 2 warm-up rounds, 5 timed):
 *   ZNN_STRATEGY_DIRECT    the direct method in all three passes
 *   ZNN_STRATEGY_FFT       the FFT method, every pass transforms what it needs
 *   ZNN_STRATEGY_FFT_MEMO  the FFT method with the kernels transformed once per
 *                          round and shared by forward and backward
 *                          (znn_conv_prepare_kernels) and with the node spectra
 *                          of forward and backward kept for the kernel gradient
 *                          (znn_conv_set_memo + znn_conv3d_wgrad_memo)
 * bytes[t] is the device memory strategy t holds during a round beyond the
 * layer's own tensors (workspace, kernel spectra, memoized node spectra).  A
 * strategy whose bytes exceed memory_budget is not run (ms[t] = INFINITY) and
 * cannot be chosen; ZNN_EWORKSPACE if none fits.  `chosen` is the fastest one
 * that ran; its method (direct / FFT) is also stored in the cache that
 * ZNN_AUTO plans consult.  `ws` must hold the layer's tensors plus the largest
 * strategy that fits the budget; znn_autotune_round_workspace_bytes returns
 * that size for an unlimited budget, which is always enough.  Synchronises
 * `stream` with the host.
 */
typedef enum znn_strategy {
    ZNN_STRATEGY_DIRECT   = 0,
    ZNN_STRATEGY_FFT      = 1,
    ZNN_STRATEGY_FFT_MEMO = 2
} znn_strategy;

typedef struct znn_round_report {
    float    ms[3];      /* mean milliseconds per round, indexed by znn_strategy */
    uint64_t bytes[3];   /* device bytes held during a round, indexed by znn_strategy */
    int32_t  chosen;     /* znn_strategy */
} znn_round_report;

int  znn_autotune_round_workspace_bytes(const znn_conv_desc* desc, size_t* bytes);
int  znn_autotune_round(const znn_conv_desc* desc, uint64_t memory_budget, void* ws, size_t ws_bytes,
                        void* stream, znn_round_report* report);

/*
 * Kernel-level timing for benchmarks and roofline reports.  While enabled, every
 * kernel the library launches is bracketed by two HIP events on its stream.
 * znn_trace_collect waits for the recorded launches, returns them in launch
 * order (name of the kernel's role, milliseconds) and forgets them; *count is
 * the number recorded even when it exceeds `capacity`.  Process-wide; off by default.
 */
typedef struct { char name[56]; float ms; } znn_trace_record;
int  znn_trace_enable(int32_t on);
int  znn_trace_collect(znn_trace_record* records, int32_t capacity, int32_t* count);

/* Description of the last error on the calling thread ("" if none). Never NULL. */
const char* znn_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ZNN_H */
