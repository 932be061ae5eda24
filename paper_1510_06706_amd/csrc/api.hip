// Host side of the C ABI: validation, plans, dispatch, autotuner cache.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <tuple>
#include <vector>

#include "znn_internal.h"

#include <algorithm>

namespace znn {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int check_launch(const char* what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ZNN_EHIP, "%s: %s", what, hipGetErrorString(e));
    return ZNN_OK;
}

// ---------------------------------------------------------------- tracing
struct TraceEntry { const char* name; hipEvent_t e0, e1; };
static std::mutex g_trace_mu;
static bool g_trace_on = false;
static std::vector<TraceEntry> g_trace;

TraceScope::TraceScope(const char* name, hipStream_t s) : slot(-1), stream(s)
{
    if (!g_trace_on) return;
    std::lock_guard<std::mutex> lk(g_trace_mu);
    TraceEntry e;
    e.name = name;
    if (hipEventCreate(&e.e0) != hipSuccess) return;
    if (hipEventCreate(&e.e1) != hipSuccess) { (void)hipEventDestroy(e.e0); return; }
    (void)hipEventRecord(e.e0, s);
    g_trace.push_back(e);
    slot = (int)g_trace.size() - 1;
}

TraceScope::~TraceScope()
{
    if (slot < 0) return;
    std::lock_guard<std::mutex> lk(g_trace_mu);
    if (slot < (int)g_trace.size()) (void)hipEventRecord(g_trace[slot].e1, stream);
}

const Tuning& tuning()
{
    static const Tuning t = [] {
        auto flag = [](const char* name) { const char* e = getenv(name); return e && *e && *e != '0'; };
        auto num = [](const char* name, int dflt) { const char* e = getenv(name); return e && *e ? atoi(e) : dflt; };
        Tuning v = {};
        v.log = flag("ZNN_LOG");
        v.conv_u1 = flag("ZNN_CONV_U1");
        v.conv_no_wl = flag("ZNN_CONV_NO_WL");
        v.conv_no_split = flag("ZNN_CONV_NO_SPLIT");
        v.conv_no_tail = flag("ZNN_CONV_NO_TAIL");
        if (const char* e = getenv("ZNN_CONV_TILE"))
            if (sscanf(e, "%d,%d,%d,%d", &v.conv_tile[0], &v.conv_tile[1], &v.conv_tile[2], &v.conv_tile[3]) != 4)
                v.conv_tile[0] = v.conv_tile[1] = v.conv_tile[2] = v.conv_tile[3] = 0;
        v.wgrad_halves = num("ZNN_WGRAD_HALVES", 2);
        v.wgrad_maxnj = num("ZNN_WGRAD_MAXNJ", 6);
        if (v.wgrad_maxnj < 1 || v.wgrad_maxnj > 8) v.wgrad_maxnj = 6;
        v.wgrad_own_columns_from = num("ZNN_WGRAD_OWN_COLUMNS_FROM", 16);
        v.wgrad_own_waves = num("ZNN_WGRAD_OWN_WAVES", 4) == 8 ? 8 : 4;
        v.wgrad_stride_mod = num("ZNN_WGRAD_STRIDE_MOD", 4);
        if (v.wgrad_stride_mod < 0 || v.wgrad_stride_mod > 28 || v.wgrad_stride_mod % 4) v.wgrad_stride_mod = 4;
        v.wgrad_slow_loader = flag("ZNN_WGRAD_SLOW_LOADER");
        v.fft_mac_z0 = num("ZNN_FFT_MAC_Z0", 0);
        v.fft_mac_valu = flag("ZNN_FFT_MAC_VALU");
        v.fft_wgrad_plain = flag("ZNN_FFT_WGRAD_PLAIN");
        v.fft_no_taps_pass = flag("ZNN_FFT_NO_TAPS_PASS");
        v.fft_no_two_level = flag("ZNN_FFT_NO_TWO_LEVEL");
        v.fft_no_mac_inverse = flag("ZNN_FFT_NO_MAC_INVERSE");
        v.fft_lds_kb = num("ZNN_FFT_LDS_KB", 0);
        if (v.fft_lds_kb < 8 || v.fft_lds_kb > 64) v.fft_lds_kb = 0;
        v.fft_no_fused_xy = flag("ZNN_FFT_NO_FUSED_XY");
        v.fft_lds_passes = flag("ZNN_FFT_LDS_PASSES");
        return v;
    }();
    return t;
}

int next_fft_extent(int n)
{
    for (int m = n;; ++m) {
        int t = m;
        while (t % 2 == 0) t /= 2;
        while (t % 3 == 0) t /= 3;
        while (t % 5 == 0) t /= 5;
        if (t == 1) return m;
    }
}

// ---------------------------------------------------------------- autotune cache
using DescKey = std::tuple<int, int, int, int, int, int, int, int, int, int, int>;
static std::mutex g_tune_mu;
static std::map<DescKey, int> g_tune;

static DescKey key_of(const znn_conv_desc& d)
{
    return DescKey(d.fan_in, d.fan_out, d.image.z, d.image.y, d.image.x, d.kernel.z, d.kernel.y, d.kernel.x,
                   d.sparsity.z, d.sparsity.y, d.sparsity.x);
}

// Cost model behind mode = auto when no measurement is cached, calibrated on the five
// benchmark configurations and the layers of the benchmark networks.  Direct: a dense fp32
// contraction at about 92 effective TFLOP/s, scaled down when the output has too few voxel
// tiles (times the shares its input maps can be split into) to occupy the 256 compute units.  FFT: the two multiply-accumulates and the pruned
// DFTs of the kernel gradient are ALU work (kernel taps folded in) or stream the full kernel
// spectra from HBM (small layers, extents not divisible by 4), the node transforms move
// 16 bytes per frequency and pass at about 3.5 TB/s effective; both pay per launch.
static int model_choice(const Geom& g)
{
    const double macs = (double)g.f * g.fo * (double)g.ovol() * (double)g.kvol();
    const double tiles = std::ceil((double)g.ovol() / 128.0) * std::ceil((double)g.fo / 128.0);
    const double nchunk = std::ceil(g.f / 4.0);
    const double splits = tiles >= 256.0 ? 1.0 : std::min(nchunk, std::ceil(768.0 / tiles));
    const double util = std::min(1.0, tiles * splits / 1024.0);
    const double t_direct = 3.0 * 2.0 * macs / (92e12 * util) + 7 * 10e-6;
    const double sv = (double)g.svol();
    const double pairs = (double)g.f * g.fo;
    const int taps = g.Nz > 1 ? g.kz : g.ky;
    const int N = g.Nz > 1 ? g.Nz : g.Ny;
    const int sp = g.Nz > 1 ? g.spz : g.spy;
    const double P = g.Nz > 1 ? (double)g.Ny * g.Nxh : (double)g.Nxh;
    const double mac_blocks = std::ceil(P / 64.0) * std::ceil(N / 32.0) * std::ceil(std::min(g.f, g.fo) / 4.0);
    const bool folded = N % 4 == 0 && taps <= 16 && taps < N && sp == 1 && mac_blocks >= 128.0;
    double t_mac;
    // the folded multiply-accumulate needs about four workgroups per compute unit to reach its rate
    if (folded) t_mac = 2.0 * 8.0 * taps * sv * pairs / (55e12 * std::min(1.0, mac_blocks / 1024.0)) + 8.0 * taps * P * pairs / 3e12;
    else t_mac = 8.0 * sv * pairs * (1.0 / 4.5e12 + 2.0 / 5.5e12 + 0.3 / 5e12);
    const double t_dft = (taps / 4.0 + 2.0) * 8.0 * sv * pairs / 45e12;
    const double t_nodes = 3.0 * (g.f + g.fo) * 3.0 * 16.0 * sv / 3.5e12;
    const double t_fft = t_mac + t_dft + t_nodes + 25 * 6e-6;
    return t_fft < t_direct ? ZNN_FFT : ZNN_DIRECT;
}

static int validate_desc(const znn_conv_desc* d, Geom* g)
{
    if (!d) return fail(ZNN_EINVAL, "descriptor is NULL");
    if (d->fan_in < 1 || d->fan_out < 1)
        return fail(ZNN_EINVAL, "fan_in and fan_out must be >= 1 (got %d, %d)", d->fan_in, d->fan_out);
    const int n[3] = {d->image.z, d->image.y, d->image.x};
    const int k[3] = {d->kernel.z, d->kernel.y, d->kernel.x};
    const int sp[3] = {d->sparsity.z, d->sparsity.y, d->sparsity.x};
    for (int a = 0; a < 3; ++a) {
        if (n[a] < 1 || k[a] < 1) return fail(ZNN_EINVAL, "image and kernel extents must be >= 1");
        if (sp[a] < 1) return fail(ZNN_EINVAL, "sparsity must be >= 1");
        if ((long)sp[a] * (k[a] - 1) + 1 > n[a])
            return fail(ZNN_EINVAL, "kernel extent %d (sparsity %d) exceeds image extent %d on axis %d",
                        k[a], sp[a], n[a], a);
    }
    if (d->mode != ZNN_DIRECT && d->mode != ZNN_FFT && d->mode != ZNN_AUTO)
        return fail(ZNN_EINVAL, "unknown mode %d", d->mode);
    g->f = d->fan_in; g->fo = d->fan_out;
    g->nz = n[0]; g->ny = n[1]; g->nx = n[2];
    g->kz = k[0]; g->ky = k[1]; g->kx = k[2];
    g->spz = sp[0]; g->spy = sp[1]; g->spx = sp[2];
    g->oz = n[0] - sp[0] * (k[0] - 1); g->oy = n[1] - sp[1] * (k[1] - 1); g->ox = n[2] - sp[2] * (k[2] - 1);
    if ((double)g->nvol() >= 2147483648.0)
        return fail(ZNN_EUNSUPPORTED, "image volume does not fit 32-bit voxel offsets");
    g->Nz = next_fft_extent(n[0]); g->Ny = next_fft_extent(n[1]); g->Nx = next_fft_extent(n[2]);
    g->Nxh = g->Nx / 2 + 1;
    return ZNN_OK;
}

static bool aligned256(const void* p) { return ((uintptr_t)p & 255) == 0; }

static int check_ws(const znn_plan* p, int pass, void* ws, size_t ws_bytes)
{
    size_t need = 0;
    int rc = znn_plan_workspace_bytes(p, pass, &need);
    if (rc != ZNN_OK) return rc;
    if (need == 0) return ZNN_OK;
    if (!ws) return fail(ZNN_EWORKSPACE, "workspace is NULL but %zu bytes are needed", need);
    if (!aligned256(ws)) return fail(ZNN_EWORKSPACE, "workspace is not 256-byte aligned");
    if (ws_bytes < need) return fail(ZNN_EWORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, need);
    return ZNN_OK;
}

}  // namespace znn

using namespace znn;

extern "C" {

const char* znn_last_error(void) { return g_err; }

int znn_trace_enable(int32_t on)
{
    std::lock_guard<std::mutex> lk(g_trace_mu);
    g_trace_on = on != 0;
    return ZNN_OK;
}

int znn_trace_collect(znn_trace_record* records, int32_t capacity, int32_t* count)
{
    if (!count || capacity < 0 || (capacity > 0 && !records)) return fail(ZNN_EINVAL, "bad trace buffer");
    std::lock_guard<std::mutex> lk(g_trace_mu);
    int n = 0, rc = ZNN_OK;
    for (TraceEntry& e : g_trace) {
        float ms = 0.f;
        if (hipEventSynchronize(e.e1) != hipSuccess || hipEventElapsedTime(&ms, e.e0, e.e1) != hipSuccess)
            rc = fail(ZNN_EHIP, "cannot read the events of '%s'", e.name);
        if (n < capacity) {
            snprintf(records[n].name, sizeof(records[n].name), "%s", e.name);
            records[n].ms = ms;
        }
        ++n;
        (void)hipEventDestroy(e.e0);
        (void)hipEventDestroy(e.e1);
    }
    g_trace.clear();
    *count = n;
    return rc;
}

int znn_plan_create(const znn_conv_desc* desc, znn_plan** plan)
{
    if (!plan) return fail(ZNN_EINVAL, "plan output pointer is NULL");
    Geom g;
    int rc = validate_desc(desc, &g);
    if (rc != ZNN_OK) return rc;
    int mode = desc->mode;
    if (mode == ZNN_AUTO) {
        std::lock_guard<std::mutex> lk(g_tune_mu);
        auto it = g_tune.find(key_of(*desc));
        mode = (it != g_tune.end()) ? it->second : model_choice(g);
        if (mode == ZNN_FFT && (g.Nz > kMaxFftExtent || g.Ny > kMaxFftExtent || g.Nx > kMaxFftExtent))
            mode = ZNN_DIRECT;
    }
    if (mode == ZNN_FFT && (g.Nz > kMaxFftExtent || g.Ny > kMaxFftExtent || g.Nx > kMaxFftExtent))
        return fail(ZNN_EUNSUPPORTED, "FFT extents above %d are not supported", kMaxFftExtent);
    znn_plan* p = new (std::nothrow) znn_plan;
    if (!p) return fail(ZNN_EINVAL, "out of host memory");
    p->desc = *desc;
    p->g = g;
    p->mode = mode;
    p->fold = mode == ZNN_FFT ? fold_default(g) : fold_full();
    p->resident = nullptr;
    p->memo = nullptr;
    p->memo_has_in = p->memo_has_gout = false;
    *plan = p;
    return ZNN_OK;
}

void znn_plan_destroy(znn_plan* plan) { delete plan; }

int znn_plan_mode(const znn_plan* plan, int32_t* mode)
{
    if (!plan || !mode) return fail(ZNN_EINVAL, "NULL argument");
    *mode = plan->mode;
    return ZNN_OK;
}

int znn_plan_fft_extents(const znn_plan* plan, znn_vec3* N)
{
    if (!plan || !N) return fail(ZNN_EINVAL, "NULL argument");
    N->z = plan->g.Nz; N->y = plan->g.Ny; N->x = plan->g.Nx;
    return ZNN_OK;
}

int znn_plan_workspace_bytes(const znn_plan* plan, int32_t pass, size_t* bytes)
{
    if (!plan || !bytes) return fail(ZNN_EINVAL, "NULL argument");
    if (pass < ZNN_PASS_FWD || pass > ZNN_PASS_WGRAD) return fail(ZNN_EINVAL, "unknown pass %d", pass);
    if (plan->mode == ZNN_DIRECT) *bytes = direct_workspace_bytes(plan->g, pass);
    else *bytes = fft_workspace(plan->g, plan->fold, pass, plan->resident != nullptr).total;
    return ZNN_OK;
}

int znn_plan_spectra_bytes(const znn_plan* plan, size_t* bytes)
{
    if (!plan || !bytes) return fail(ZNN_EINVAL, "NULL argument");
    *bytes = fft_spectra_bytes(plan->g, plan->fold);
    return ZNN_OK;
}

int znn_plan_spectra_layout(const znn_plan* plan, int32_t* layout)
{
    if (!plan || !layout) return fail(ZNN_EINVAL, "NULL argument");
    *layout = plan->fold.on ? ZNN_SPECTRA_FOLDED : ZNN_SPECTRA_FULL;
    return ZNN_OK;
}

int znn_plan_set_spectra_layout(znn_plan* plan, int32_t layout)
{
    if (!plan) return fail(ZNN_EINVAL, "NULL argument");
    if (plan->mode != ZNN_FFT) return fail(ZNN_EINVAL, "kernel spectra exist only for the FFT method");
    if (plan->resident)
        return fail(ZNN_EINVAL, "resident kernel spectra are attached in the current layout; release them first");
    if (layout == ZNN_SPECTRA_AUTO) plan->fold = fold_default(plan->g);
    else if (layout == ZNN_SPECTRA_FULL) plan->fold = fold_full();
    else if (layout == ZNN_SPECTRA_FOLDED) {
        const Fold F = fold_forced(plan->g);
        if (!F.on)
            return fail(ZNN_EUNSUPPORTED, "half spectra need a slowest axis whose FFT extent is divisible by 4 "
                                          "with at most %d taps one voxel apart", kMaxFoldedTaps);
        plan->fold = F;
    } else return fail(ZNN_EINVAL, "unknown spectra layout %d", layout);
    return ZNN_OK;
}

int znn_conv_prepare_kernels(znn_plan* plan, const float* w, void* spectra, size_t spectra_bytes,
                             void* ws, size_t ws_bytes, void* stream)
{
    (void)ws; (void)ws_bytes;
    if (!plan || !w) return fail(ZNN_EINVAL, "NULL argument");
    if (plan->mode != ZNN_FFT) return fail(ZNN_EINVAL, "kernel spectra exist only for the FFT method");
    const size_t need = fft_spectra_bytes(plan->g, plan->fold);
    if (!spectra) return fail(ZNN_EWORKSPACE, "spectra buffer is NULL");
    if (!aligned256(spectra)) return fail(ZNN_EWORKSPACE, "spectra buffer is not 256-byte aligned");
    if (spectra_bytes < need) return fail(ZNN_EWORKSPACE, "spectra buffer has %zu bytes, %zu needed", spectra_bytes, need);
    int rc = fft_kernel_spectra(plan->g, plan->fold, w, (float2*)spectra, (hipStream_t)stream);
    if (rc != ZNN_OK) return rc;
    plan->resident = (const float2*)spectra;
    return ZNN_OK;
}

int znn_plan_memo_bytes(const znn_plan* plan, size_t* bytes)
{
    if (!plan || !bytes) return fail(ZNN_EINVAL, "NULL argument");
    *bytes = align256(sizeof(float2) * (size_t)(plan->g.f + plan->g.fo) * plan->g.svol());
    return ZNN_OK;
}

int znn_conv_set_memo(znn_plan* plan, void* memo, size_t memo_bytes)
{
    if (!plan) return fail(ZNN_EINVAL, "NULL argument");
    plan->memo = nullptr;
    plan->memo_has_in = plan->memo_has_gout = false;
    if (!memo) return ZNN_OK;
    if (plan->mode != ZNN_FFT) return fail(ZNN_EINVAL, "spectra are memoized only by the FFT method");
    size_t need = 0;
    znn_plan_memo_bytes(plan, &need);
    if (!aligned256(memo)) return fail(ZNN_EWORKSPACE, "memo buffer is not 256-byte aligned");
    if (memo_bytes < need) return fail(ZNN_EWORKSPACE, "memo buffer has %zu bytes, %zu needed", memo_bytes, need);
    plan->memo = (float2*)memo;
    return ZNN_OK;
}

int znn_conv3d_wgrad_memo(znn_plan* plan, float* gw, void* ws, size_t ws_bytes, void* stream)
{
    if (!plan || !gw) return fail(ZNN_EINVAL, "NULL argument");
    if (plan->mode != ZNN_FFT || !plan->memo) return fail(ZNN_EINVAL, "no memo buffer is attached to this plan");
    if (!plan->memo_has_in || !plan->memo_has_gout)
        return fail(ZNN_EINVAL, "the forward and the backward pass must run on this plan first");
    int rc = check_ws(plan, ZNN_PASS_WGRAD, ws, ws_bytes);
    if (rc != ZNN_OK) return rc;
    const float2* Ihat = plan->memo;
    const float2* Ghat = plan->memo + (size_t)plan->g.f * plan->g.svol();
    return fft_wgrad_from_spectra(plan->g, Ihat, Ghat, gw, ws, (hipStream_t)stream);
}

int znn_conv_release_kernels(znn_plan* plan)
{
    if (!plan) return fail(ZNN_EINVAL, "NULL argument");
    plan->resident = nullptr;
    return ZNN_OK;
}

int znn_conv3d_fwd(znn_plan* plan, const float* in, const float* w, float* out,
                   void* ws, size_t ws_bytes, void* stream)
{
    if (!plan || !in || !out) return fail(ZNN_EINVAL, "NULL argument");
    if (!w && !(plan->mode == ZNN_FFT && plan->resident)) return fail(ZNN_EINVAL, "kernel pointer is NULL");
    int rc = check_ws(plan, ZNN_PASS_FWD, ws, ws_bytes);
    if (rc != ZNN_OK) return rc;
    if (plan->mode == ZNN_DIRECT) return direct_fwd(plan->g, in, w, out, ws, (hipStream_t)stream);
    rc = fft_fwd(plan->g, plan->fold, in, w, plan->resident, out, ws, plan->memo, (hipStream_t)stream);
    if (plan->memo) plan->memo_has_in = rc == ZNN_OK;
    return rc;
}

int znn_conv3d_bwd(znn_plan* plan, const float* gout, const float* w, float* gin,
                   void* ws, size_t ws_bytes, void* stream)
{
    if (!plan || !gout || !gin) return fail(ZNN_EINVAL, "NULL argument");
    if (!w && !(plan->mode == ZNN_FFT && plan->resident)) return fail(ZNN_EINVAL, "kernel pointer is NULL");
    int rc = check_ws(plan, ZNN_PASS_BWD, ws, ws_bytes);
    if (rc != ZNN_OK) return rc;
    if (plan->mode == ZNN_DIRECT) return direct_bwd(plan->g, gout, w, gin, ws, (hipStream_t)stream);
    rc = fft_bwd(plan->g, plan->fold, gout, w, plan->resident, gin, ws,
                 plan->memo ? plan->memo + (size_t)plan->g.f * plan->g.svol() : nullptr, (hipStream_t)stream);
    if (plan->memo) plan->memo_has_gout = rc == ZNN_OK;
    return rc;
}

int znn_conv3d_wgrad(znn_plan* plan, const float* in, const float* gout, float* gw,
                     void* ws, size_t ws_bytes, void* stream)
{
    if (!plan || !in || !gout || !gw) return fail(ZNN_EINVAL, "NULL argument");
    int rc = check_ws(plan, ZNN_PASS_WGRAD, ws, ws_bytes);
    if (rc != ZNN_OK) return rc;
    if (plan->mode == ZNN_DIRECT) return direct_wgrad(plan->g, in, gout, gw, ws, (hipStream_t)stream);
    return fft_wgrad(plan->g, in, gout, gw, ws, (hipStream_t)stream);
}

// ---------------------------------------------------------------- autotuner
static size_t tune_tensor_bytes(const Geom& g, size_t off[6])
{
    size_t o = 0;
    off[0] = o; o += align256(sizeof(float) * g.f * g.nvol());                 // in
    off[1] = o; o += align256(sizeof(float) * g.fo * g.f * g.kvol());          // w
    off[2] = o; o += align256(sizeof(float) * g.fo * g.ovol());                // gout
    off[3] = o; o += align256(sizeof(float) * g.f * g.nvol());                 // gin
    off[4] = o; o += align256(sizeof(float) * g.fo * g.f * g.kvol());          // gw
    off[5] = o; o += align256(sizeof(float) * g.fo * g.ovol());                // out
    return o;
}

static size_t tune_scratch_bytes(const Geom& g, bool fft_ok)
{
    const Fold F = fold_default(g);
    size_t m = 0;
    for (int pass = 0; pass < 3; ++pass) {
        size_t d = direct_workspace_bytes(g, pass);
        if (d > m) m = d;
        if (fft_ok) {
            size_t f = fft_workspace(g, F, pass, false).total;
            if (f > m) m = f;
        }
    }
    return m;
}

int znn_autotune_workspace_bytes(const znn_conv_desc* desc, size_t* bytes)
{
    if (!bytes) return fail(ZNN_EINVAL, "NULL argument");
    Geom g;
    int rc = validate_desc(desc, &g);
    if (rc != ZNN_OK) return rc;
    const bool fft_ok = g.Nz <= kMaxFftExtent && g.Ny <= kMaxFftExtent && g.Nx <= kMaxFftExtent;
    size_t off[6];
    *bytes = tune_tensor_bytes(g, off) + tune_scratch_bytes(g, fft_ok);
    return ZNN_OK;
}

int znn_autotune(const znn_conv_desc* desc, void* ws, size_t ws_bytes, void* stream,
                 int32_t* chosen_mode, float ms[2][3])
{
    if (!chosen_mode || !ms) return fail(ZNN_EINVAL, "NULL argument");
    Geom g;
    int rc = validate_desc(desc, &g);
    if (rc != ZNN_OK) return rc;
    const bool fft_ok = g.Nz <= kMaxFftExtent && g.Ny <= kMaxFftExtent && g.Nx <= kMaxFftExtent;
    size_t off[6];
    const size_t tensors = tune_tensor_bytes(g, off);
    const size_t scratch = tune_scratch_bytes(g, fft_ok);
    if (!ws) return fail(ZNN_EWORKSPACE, "workspace is NULL");
    if (!aligned256(ws)) return fail(ZNN_EWORKSPACE, "workspace is not 256-byte aligned");
    if (ws_bytes < tensors + scratch)
        return fail(ZNN_EWORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, tensors + scratch);
    hipStream_t s = (hipStream_t)stream;
    char* base = (char*)ws;
    float* in = (float*)(base + off[0]);
    float* w = (float*)(base + off[1]);
    float* gout = (float*)(base + off[2]);
    float* gin = (float*)(base + off[3]);
    float* gw = (float*)(base + off[4]);
    float* out = (float*)(base + off[5]);
    void* scr = base + tensors;
    if ((rc = fill_pattern(in, (long)g.f * g.nvol(), 1.0f, s)) != ZNN_OK) return rc;
    if ((rc = fill_pattern(w, (long)g.fo * g.f * g.kvol(), 1.0f / std::sqrt((float)(g.f * g.kvol())), s)) != ZNN_OK) return rc;
    if ((rc = fill_pattern(gout, (long)g.fo * g.ovol(), 1.0f, s)) != ZNN_OK) return rc;

    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)
        return fail(ZNN_EHIP, "hipEventCreate failed");
    const int warm = 2, timed = 5;
    const Fold F = fold_default(g);
    for (int m = 0; m < 2; ++m)
        for (int p = 0; p < 3; ++p) ms[m][p] = INFINITY;
    rc = ZNN_OK;
    for (int mode = 0; mode < 2 && rc == ZNN_OK; ++mode) {
        if (mode == ZNN_FFT && !fft_ok) continue;
        for (int pass = 0; pass < 3 && rc == ZNN_OK; ++pass) {
            for (int it = 0; it < warm + timed && rc == ZNN_OK; ++it) {
                if (it == warm) (void)hipEventRecord(e0, s);
                if (mode == ZNN_DIRECT) {
                    if (pass == 0) rc = direct_fwd(g, in, w, out, scr, s);
                    else if (pass == 1) rc = direct_bwd(g, gout, w, gin, scr, s);
                    else rc = direct_wgrad(g, in, gout, gw, scr, s);
                } else {
                    if (pass == 0) rc = fft_fwd(g, F, in, w, nullptr, out, scr, nullptr, s);
                    else if (pass == 1) rc = fft_bwd(g, F, gout, w, nullptr, gin, scr, nullptr, s);
                    else rc = fft_wgrad(g, in, gout, gw, scr, s);
                }
            }
            if (rc != ZNN_OK) break;
            (void)hipEventRecord(e1, s);
            if (hipEventSynchronize(e1) != hipSuccess) { rc = fail(ZNN_EHIP, "hipEventSynchronize failed"); break; }
            float t = 0.f;
            (void)hipEventElapsedTime(&t, e0, e1);
            ms[mode][pass] = t / timed;
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != ZNN_OK) return rc;
    const float td = ms[0][0] + ms[0][1] + ms[0][2];
    const float tf = ms[1][0] + ms[1][1] + ms[1][2];
    const int choice = (fft_ok && tf < td) ? ZNN_FFT : ZNN_DIRECT;
    {
        std::lock_guard<std::mutex> lk(g_tune_mu);
        g_tune[key_of(*desc)] = choice;
    }
    *chosen_mode = choice;
    return ZNN_OK;
}

// ---- whole-round strategies under a memory budget (Section 4, memoization)
struct RoundNeeds {
    size_t scratch[3];      // workspace, kernel spectra, memoized node spectra per strategy (summed below)
    size_t total[3];
};

static RoundNeeds round_needs(const Geom& g, bool fft_ok)
{
    RoundNeeds r = {};
    const Fold F = fold_default(g);
    size_t d = 0, f = 0, fm = 0;
    for (int pass = 0; pass < 3; ++pass) {
        d = std::max(d, direct_workspace_bytes(g, pass));
        if (fft_ok) {
            f = std::max(f, fft_workspace(g, F, pass, false).total);
            fm = std::max(fm, fft_workspace(g, F, pass, true).total);
        }
    }
    r.total[ZNN_STRATEGY_DIRECT] = d;
    r.total[ZNN_STRATEGY_FFT] = f;
    r.total[ZNN_STRATEGY_FFT_MEMO] = fft_ok
        ? fm + fft_spectra_bytes(g, F) + align256(sizeof(float2) * (size_t)(g.f + g.fo) * g.svol()) : 0;
    return r;
}

int znn_autotune_round_workspace_bytes(const znn_conv_desc* desc, size_t* bytes)
{
    if (!bytes) return fail(ZNN_EINVAL, "NULL argument");
    Geom g;
    int rc = validate_desc(desc, &g);
    if (rc != ZNN_OK) return rc;
    const bool fft_ok = g.Nz <= kMaxFftExtent && g.Ny <= kMaxFftExtent && g.Nx <= kMaxFftExtent;
    const RoundNeeds need = round_needs(g, fft_ok);
    size_t off[6];
    *bytes = tune_tensor_bytes(g, off) + std::max(need.total[0], std::max(need.total[1], need.total[2]));
    return ZNN_OK;
}

int znn_autotune_round(const znn_conv_desc* desc, uint64_t memory_budget, void* ws, size_t ws_bytes,
                       void* stream, znn_round_report* report)
{
    if (!report) return fail(ZNN_EINVAL, "NULL argument");
    Geom g;
    int rc = validate_desc(desc, &g);
    if (rc != ZNN_OK) return rc;
    const bool fft_ok = g.Nz <= kMaxFftExtent && g.Ny <= kMaxFftExtent && g.Nx <= kMaxFftExtent;
    const RoundNeeds need = round_needs(g, fft_ok);
    bool run[3];
    size_t scratch = 0;
    int candidates = 0;
    for (int t = 0; t < 3; ++t) {
        report->ms[t] = INFINITY;
        report->bytes[t] = need.total[t];
        run[t] = (t == ZNN_STRATEGY_DIRECT || fft_ok) && need.total[t] <= memory_budget;
        if (run[t]) { scratch = std::max(scratch, need.total[t]); ++candidates; }
    }
    report->chosen = -1;
    if (!candidates)
        return fail(ZNN_EWORKSPACE, "no strategy fits the memory budget of %llu bytes (direct needs %zu)",
                    (unsigned long long)memory_budget, need.total[0]);
    size_t off[6];
    const size_t tensors = tune_tensor_bytes(g, off);
    if (!ws) return fail(ZNN_EWORKSPACE, "workspace is NULL");
    if (!aligned256(ws)) return fail(ZNN_EWORKSPACE, "workspace is not 256-byte aligned");
    if (ws_bytes < tensors + scratch)
        return fail(ZNN_EWORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, tensors + scratch);
    hipStream_t s = (hipStream_t)stream;
    char* base = (char*)ws;
    float* in = (float*)(base + off[0]);
    float* w = (float*)(base + off[1]);
    float* gout = (float*)(base + off[2]);
    float* gin = (float*)(base + off[3]);
    float* gw = (float*)(base + off[4]);
    float* out = (float*)(base + off[5]);
    char* scr = base + tensors;
    if ((rc = fill_pattern(in, (long)g.f * g.nvol(), 1.0f, s)) != ZNN_OK) return rc;
    if ((rc = fill_pattern(w, (long)g.fo * g.f * g.kvol(), 1.0f / std::sqrt((float)(g.f * g.kvol())), s)) != ZNN_OK) return rc;
    if ((rc = fill_pattern(gout, (long)g.fo * g.ovol(), 1.0f, s)) != ZNN_OK) return rc;
    // memoized strategy: [pass workspace | kernel spectra | node spectra]
    const Fold F = fold_default(g);
    size_t memo_ws = 0;
    if (fft_ok)
        for (int pass = 0; pass < 3; ++pass) memo_ws = std::max(memo_ws, fft_workspace(g, F, pass, true).total);
    float2* What = (float2*)(scr + memo_ws);
    float2* Ihat = (float2*)(scr + memo_ws + fft_spectra_bytes(g, F));
    float2* Ghat = Ihat + (size_t)g.f * g.svol();

    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)
        return fail(ZNN_EHIP, "hipEventCreate failed");
    const int warm = 2, timed = 5;
    for (int t = 0; t < 3 && rc == ZNN_OK; ++t) {
        if (!run[t]) continue;
        for (int it = 0; it < warm + timed && rc == ZNN_OK; ++it) {
            if (it == warm) (void)hipEventRecord(e0, s);
            if (t == ZNN_STRATEGY_DIRECT) {
                rc = direct_fwd(g, in, w, out, scr, s);
                if (rc == ZNN_OK) rc = direct_bwd(g, gout, w, gin, scr, s);
                if (rc == ZNN_OK) rc = direct_wgrad(g, in, gout, gw, scr, s);
            } else if (t == ZNN_STRATEGY_FFT) {
                rc = fft_fwd(g, F, in, w, nullptr, out, scr, nullptr, s);
                if (rc == ZNN_OK) rc = fft_bwd(g, F, gout, w, nullptr, gin, scr, nullptr, s);
                if (rc == ZNN_OK) rc = fft_wgrad(g, in, gout, gw, scr, s);
            } else {
                rc = fft_kernel_spectra(g, F, w, What, s);
                if (rc == ZNN_OK) rc = fft_fwd(g, F, in, nullptr, What, out, scr, Ihat, s);
                if (rc == ZNN_OK) rc = fft_bwd(g, F, gout, nullptr, What, gin, scr, Ghat, s);
                if (rc == ZNN_OK) rc = fft_wgrad_from_spectra(g, Ihat, Ghat, gw, scr, s);
            }
        }
        if (rc != ZNN_OK) break;
        (void)hipEventRecord(e1, s);
        if (hipEventSynchronize(e1) != hipSuccess) { rc = fail(ZNN_EHIP, "hipEventSynchronize failed"); break; }
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, e0, e1);
        report->ms[t] = ms / timed;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != ZNN_OK) return rc;
    int best = -1;
    for (int t = 0; t < 3; ++t)
        if (run[t] && (best < 0 || report->ms[t] < report->ms[best])) best = t;
    report->chosen = best;
    {
        std::lock_guard<std::mutex> lk(g_tune_mu);
        g_tune[key_of(*desc)] = best == ZNN_STRATEGY_DIRECT ? ZNN_DIRECT : ZNN_FFT;
    }
    return ZNN_OK;
}

}  // extern "C"
