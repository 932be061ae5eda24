// Max-filtering and its Jacobian, the transfer-function edges, and the small
// elementwise / reduction steps of a training round.
#include "znn_internal.h"

namespace znn {

// Max-filtering (Section 2).  The window is scanned in ascending flat input
// offset with a strict '>' so the smallest offset wins among equal values.
// The window's taps lie (sz,sy,sx) voxels apart (1 = the dense filter).
__global__ void __launch_bounds__(256)
k_maxfilter_fwd(int maps, int nz, int ny, int nx, int wz, int wy, int wx, int sz, int sy, int sx,
                const float* __restrict__ in, float* __restrict__ out, int* __restrict__ idx)
{
    const int oz = nz - sz * (wz - 1), oy = ny - sy * (wy - 1), ox = nx - sx * (wx - 1);
    const long ovol = (long)oz * oy * ox, nvol = (long)nz * ny * nx;
    const long t = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= ovol * maps) return;
    const int m = (int)(t / ovol);
    const long p = t % ovol;
    const int x = (int)(p % ox), y = (int)((p / ox) % oy), z = (int)(p / ((long)ox * oy));
    const float* img = in + m * nvol;
    int best = (z * ny + y) * nx + x;
    float bv = img[best];
    for (int a = 0; a < wz; ++a)
        for (int b = 0; b < wy; ++b)
            for (int c = 0; c < wx; ++c) {
                const int q = ((z + sz * a) * ny + (y + sy * b)) * nx + (x + sx * c);
                const float v = img[q];
                if (v > bv) { bv = v; best = q; }
            }
    out[t] = bv;
    idx[t] = best;
}

// Max-filtering Jacobian (Section 3.1) in gather form: an input voxel q can only
// have been chosen by the windows that contain it; they are visited in
// ascending window offset, which is the order a serial scatter would add them.
__global__ void __launch_bounds__(256)
k_maxfilter_bwd(int maps, int nz, int ny, int nx, int wz, int wy, int wx, int sz, int sy, int sx,
                const float* __restrict__ gout, const int* __restrict__ idx, float* __restrict__ gin)
{
    const int oz = nz - sz * (wz - 1), oy = ny - sy * (wy - 1), ox = nx - sx * (wx - 1);
    const long ovol = (long)oz * oy * ox, nvol = (long)nz * ny * nx;
    const long t = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= nvol * maps) return;
    const int m = (int)(t / nvol);
    const int q = (int)(t % nvol);
    const int x = q % nx, y = (q / nx) % ny, z = q / (nx * ny);
    const float* g = gout + m * ovol;
    const int* id = idx + m * ovol;
    float acc = 0.f;
    // window p contains q through tap a when p = q - s a; descending taps give ascending p
    for (int a = wz - 1; a >= 0; --a) {
        const int pz = z - sz * a;
        if (pz < 0 || pz >= oz) continue;
        for (int b = wy - 1; b >= 0; --b) {
            const int py = y - sy * b;
            if (py < 0 || py >= oy) continue;
            for (int c = wx - 1; c >= 0; --c) {
                const int px = x - sx * c;
                if (px < 0 || px >= ox) continue;
                const long p = ((long)pz * oy + py) * ox + px;
                if (id[p] == q) acc += g[p];
            }
        }
    }
    gin[t] = acc;
}

// Max-pooling (Section 2): one thread per block of (pz,py,px) voxels, scanned in ascending
// flat input offset with a strict '>' (smallest offset wins among equal values).
__global__ void __launch_bounds__(256)
k_maxpool_fwd(int maps, int nz, int ny, int nx, int pz, int py, int px,
              const float* __restrict__ in, float* __restrict__ out, int* __restrict__ idx)
{
    const int oz = nz / pz, oy = ny / py, ox = nx / px;
    const long ovol = (long)oz * oy * ox, nvol = (long)nz * ny * nx;
    const long t = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= ovol * maps) return;
    const int m = (int)(t / ovol);
    const long p = t % ovol;
    const int x = (int)(p % ox), y = (int)((p / ox) % oy), z = (int)(p / ((long)ox * oy));
    const float* img = in + m * nvol;
    int best = ((z * pz) * ny + y * py) * nx + x * px;
    float bv = img[best];
    for (int a = 0; a < pz; ++a)
        for (int b = 0; b < py; ++b)
            for (int c = 0; c < px; ++c) {
                const int q = ((z * pz + a) * ny + (y * py + b)) * nx + (x * px + c);
                const float v = img[q];
                if (v > bv) { bv = v; best = q; }
            }
    out[t] = bv;
    idx[t] = best;
}

// Max-pooling Jacobian (Section 3.1) in gather form: an input voxel receives its block's
// value if it was that block's forward maximum, zero otherwise.
__global__ void __launch_bounds__(256)
k_maxpool_bwd(int maps, int nz, int ny, int nx, int pz, int py, int px,
              const float* __restrict__ gout, const int* __restrict__ idx, float* __restrict__ gin)
{
    const int oy = ny / py, ox = nx / px;
    const long ovol = (long)(nz / pz) * oy * ox, nvol = (long)nz * ny * nx;
    const long t = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= nvol * maps) return;
    const int m = (int)(t / nvol);
    const int q = (int)(t % nvol);
    const int x = q % nx, y = (q / nx) % ny, z = q / (nx * ny);
    const long p = m * ovol + ((long)(z / pz) * oy + y / py) * ox + x / px;
    gin[t] = idx[p] == q ? gout[p] : 0.f;
}

__global__ void __launch_bounds__(256)
k_transfer_fwd(long total, long voxels, const float* __restrict__ x, const float* __restrict__ bias,
               float* __restrict__ y)
{
    const long t = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= total) return;
    const float v = x[t] + bias[t / voxels];
    y[t] = v > 0.f ? v : 0.f;
}

__global__ void __launch_bounds__(256)
k_transfer_bwd(long total, const float* __restrict__ gy, const float* __restrict__ y, float* __restrict__ gx)
{
    const long t = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= total) return;
    gx[t] = y[t] > 0.f ? gy[t] : 0.f;
}

// Transfer functions other than the rectifier (Section 2): logistic and hyperbolic tangent.
// The backward edge multiplies by the derivative written through the forward output y.
template <int FN>
__global__ void __launch_bounds__(256)
k_transfer_fn_fwd(long total, long voxels, const float* __restrict__ x, const float* __restrict__ bias,
                  float* __restrict__ y)
{
    const long t = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= total) return;
    const float v = x[t] + bias[t / voxels];
    y[t] = FN == ZNN_LOGISTIC ? 1.0f / (1.0f + expf(-v)) : tanhf(v);
}

template <int FN>
__global__ void __launch_bounds__(256)
k_transfer_fn_bwd(long total, const float* __restrict__ gy, const float* __restrict__ y, float* __restrict__ gx)
{
    const long t = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= total) return;
    const float v = y[t];
    gx[t] = gy[t] * (FN == ZNN_LOGISTIC ? v * (1.0f - v) : 1.0f - v * v);
}

__global__ void __launch_bounds__(256)
k_cross_entropy_grad(long total, const float* __restrict__ y, const float* __restrict__ t_, float* __restrict__ g)
{
    const long t = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= total) return;
    const float v = y[t];
    g[t] = (v - t_[t]) / (v * (1.0f - v));
}

// One block per map; every thread sums a fixed strided subset in four independent partial
// sums (the loads of one trip are in flight together), then a fixed tree: the order of the
// additions depends on nothing but the shape.
__global__ void __launch_bounds__(1024)
k_bias_grad(long voxels, const float* __restrict__ g, float* __restrict__ gb)
{
    __shared__ float red[1024];
    const float* p = g + (long)blockIdx.x * voxels;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    for (long t = threadIdx.x; t < voxels; t += 4096) {
        a0 += p[t];
        if (t + 1024 < voxels) a1 += p[t + 1024];
        if (t + 2048 < voxels) a2 += p[t + 2048];
        if (t + 3072 < voxels) a3 += p[t + 3072];
    }
    red[threadIdx.x] = (a0 + a1) + (a2 + a3);
    __syncthreads();
    for (int s = 512; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) gb[blockIdx.x] = red[0];
}

__global__ void __launch_bounds__(256)
k_sub(long total, const float* __restrict__ a, const float* __restrict__ b, float* __restrict__ c)
{
    const long t = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < total) c[t] = a[t] - b[t];
}

__global__ void __launch_bounds__(256)
k_accumulate(long total, const float* __restrict__ x, float* __restrict__ y)
{
    const long t = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < total) y[t] = y[t] + x[t];
}

__global__ void __launch_bounds__(256)
k_sgd(long total, float eta, const float* __restrict__ g, float* __restrict__ p)
{
    const long t = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < total) p[t] = p[t] - eta * g[t];
}

// Deterministic filler for the autotuner's scratch tensors: a cheap hash of the
// element index mapped to [-scale, scale).
__global__ void __launch_bounds__(256)
k_fill_pattern(long total, float scale, float* __restrict__ p)
{
    const long t = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= total) return;
    unsigned h = (unsigned)t * 2654435761u;
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    p[t] = scale * ((float)(h >> 8) * (1.0f / 8388608.0f) - 1.0f);
}

int fill_pattern(float* p, long count, float scale, hipStream_t s)
{
    if (count <= 0) return ZNN_OK;
    ZNN_LAUNCH("fill", s, k_fill_pattern, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, count, scale, p);
    return check_launch("fill");
}

// pool = true: blocks of `win` voxels must tile the image; otherwise a sliding window whose
// taps lie `sp` voxels apart must fit inside it.
static int check_filter(int32_t maps, znn_vec3 n, znn_vec3 win, znn_vec3 sp, bool pool)
{
    if (maps < 1) return fail(ZNN_EINVAL, "maps must be >= 1");
    const int nn[3] = {n.z, n.y, n.x}, ww[3] = {win.z, win.y, win.x}, ss[3] = {sp.z, sp.y, sp.x};
    for (int a = 0; a < 3; ++a) {
        if (nn[a] < 1 || ww[a] < 1) return fail(ZNN_EINVAL, "image and window extents must be >= 1");
        if (ss[a] < 1) return fail(ZNN_EINVAL, "sparsity must be >= 1");
        if (pool) {
            if (nn[a] % ww[a] != 0)
                return fail(ZNN_EINVAL, "image extent %d is not divisible by block extent %d on axis %d", nn[a], ww[a], a);
        } else if ((long)ss[a] * (ww[a] - 1) + 1 > nn[a]) {
            return fail(ZNN_EINVAL, "window extent %d (sparsity %d) exceeds image extent %d on axis %d",
                        ww[a], ss[a], nn[a], a);
        }
    }
    if ((double)n.z * n.y * n.x >= 2147483648.0)
        return fail(ZNN_EUNSUPPORTED, "image volume does not fit int32 offsets");
    const double total = (double)maps * n.z * n.y * n.x;
    if (total / 256.0 >= 2147483647.0) return fail(ZNN_EUNSUPPORTED, "too many voxels for one launch");
    return ZNN_OK;
}

}  // namespace znn

using namespace znn;

extern "C" {

int znn_maxfilter3d_sparse_fwd(int32_t maps, znn_vec3 n, znn_vec3 win, znn_vec3 sp, const float* in,
                               float* out, int32_t* idx, void* stream)
{
    int rc = check_filter(maps, n, win, sp, false);
    if (rc != ZNN_OK) return rc;
    if (!in || !out || !idx) return fail(ZNN_EINVAL, "NULL argument");
    const long total = (long)maps * (n.z - sp.z * (win.z - 1)) * (n.y - sp.y * (win.y - 1)) * (n.x - sp.x * (win.x - 1));
    ZNN_LAUNCH("max-filter forward", (hipStream_t)stream, k_maxfilter_fwd, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       maps, n.z, n.y, n.x, win.z, win.y, win.x, sp.z, sp.y, sp.x, in, out, idx);
    return check_launch("max-filter forward");
}

int znn_maxfilter3d_sparse_bwd(int32_t maps, znn_vec3 n, znn_vec3 win, znn_vec3 sp, const float* gout,
                               const int32_t* idx, float* gin, void* stream)
{
    int rc = check_filter(maps, n, win, sp, false);
    if (rc != ZNN_OK) return rc;
    if (!gout || !idx || !gin) return fail(ZNN_EINVAL, "NULL argument");
    const long total = (long)maps * n.z * n.y * n.x;
    ZNN_LAUNCH("max-filter backward", (hipStream_t)stream, k_maxfilter_bwd, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       maps, n.z, n.y, n.x, win.z, win.y, win.x, sp.z, sp.y, sp.x, gout, idx, gin);
    return check_launch("max-filter backward");
}

int znn_maxfilter3d_fwd(int32_t maps, znn_vec3 n, znn_vec3 win, const float* in,
                        float* out, int32_t* idx, void* stream)
{
    const znn_vec3 one = {1, 1, 1};
    return znn_maxfilter3d_sparse_fwd(maps, n, win, one, in, out, idx, stream);
}

int znn_maxfilter3d_bwd(int32_t maps, znn_vec3 n, znn_vec3 win, const float* gout,
                        const int32_t* idx, float* gin, void* stream)
{
    const znn_vec3 one = {1, 1, 1};
    return znn_maxfilter3d_sparse_bwd(maps, n, win, one, gout, idx, gin, stream);
}

int znn_maxpool3d_fwd(int32_t maps, znn_vec3 n, znn_vec3 p, const float* in,
                      float* out, int32_t* idx, void* stream)
{
    const znn_vec3 one = {1, 1, 1};
    int rc = check_filter(maps, n, p, one, true);
    if (rc != ZNN_OK) return rc;
    if (!in || !out || !idx) return fail(ZNN_EINVAL, "NULL argument");
    const long total = (long)maps * (n.z / p.z) * (n.y / p.y) * (n.x / p.x);
    ZNN_LAUNCH("max-pooling forward", (hipStream_t)stream, k_maxpool_fwd, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       maps, n.z, n.y, n.x, p.z, p.y, p.x, in, out, idx);
    return check_launch("max-pooling forward");
}

int znn_maxpool3d_bwd(int32_t maps, znn_vec3 n, znn_vec3 p, const float* gout,
                      const int32_t* idx, float* gin, void* stream)
{
    const znn_vec3 one = {1, 1, 1};
    int rc = check_filter(maps, n, p, one, true);
    if (rc != ZNN_OK) return rc;
    if (!gout || !idx || !gin) return fail(ZNN_EINVAL, "NULL argument");
    const long total = (long)maps * n.z * n.y * n.x;
    ZNN_LAUNCH("max-pooling backward", (hipStream_t)stream, k_maxpool_bwd, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       maps, n.z, n.y, n.x, p.z, p.y, p.x, gout, idx, gin);
    return check_launch("max-pooling backward");
}

static int check_count(int64_t total)
{
    if (total < 1) return fail(ZNN_EINVAL, "element count must be >= 1");
    if (total / 256 >= 2147483647LL) return fail(ZNN_EUNSUPPORTED, "too many elements for one launch");
    return ZNN_OK;
}

int znn_transfer_fwd(int32_t maps, int64_t voxels, const float* x, const float* bias, float* y, void* stream)
{
    if (maps < 1 || voxels < 1) return fail(ZNN_EINVAL, "maps and voxels must be >= 1");
    if (!x || !bias || !y) return fail(ZNN_EINVAL, "NULL argument");
    const long total = (long)maps * voxels;
    int rc = check_count(total);
    if (rc != ZNN_OK) return rc;
    ZNN_LAUNCH("transfer forward", (hipStream_t)stream, k_transfer_fwd, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       total, (long)voxels, x, bias, y);
    return check_launch("transfer forward");
}

int znn_transfer_bwd(int32_t maps, int64_t voxels, const float* gy, const float* y, float* gx, void* stream)
{
    if (maps < 1 || voxels < 1) return fail(ZNN_EINVAL, "maps and voxels must be >= 1");
    if (!gy || !y || !gx) return fail(ZNN_EINVAL, "NULL argument");
    const long total = (long)maps * voxels;
    int rc = check_count(total);
    if (rc != ZNN_OK) return rc;
    ZNN_LAUNCH("transfer backward", (hipStream_t)stream, k_transfer_bwd, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       total, gy, y, gx);
    return check_launch("transfer backward");
}

int znn_transfer_fn_fwd(int32_t fn, int32_t maps, int64_t voxels, const float* x, const float* bias, float* y,
                        void* stream)
{
    if (fn == ZNN_RECTIFY) return znn_transfer_fwd(maps, voxels, x, bias, y, stream);
    if (fn != ZNN_LOGISTIC && fn != ZNN_TANH) return fail(ZNN_EINVAL, "unknown transfer function %d", fn);
    if (maps < 1 || voxels < 1) return fail(ZNN_EINVAL, "maps and voxels must be >= 1");
    if (!x || !bias || !y) return fail(ZNN_EINVAL, "NULL argument");
    const long total = (long)maps * voxels;
    int rc = check_count(total);
    if (rc != ZNN_OK) return rc;
    const dim3 grid((unsigned)((total + 255) / 256));
    if (fn == ZNN_LOGISTIC)
        ZNN_LAUNCH("transfer forward (logistic)", (hipStream_t)stream, k_transfer_fn_fwd<ZNN_LOGISTIC>, grid, dim3(256), 0,
                   total, (long)voxels, x, bias, y);
    else
        ZNN_LAUNCH("transfer forward (tanh)", (hipStream_t)stream, k_transfer_fn_fwd<ZNN_TANH>, grid, dim3(256), 0,
                   total, (long)voxels, x, bias, y);
    return check_launch("transfer forward");
}

int znn_transfer_fn_bwd(int32_t fn, int32_t maps, int64_t voxels, const float* gy, const float* y, float* gx,
                        void* stream)
{
    if (fn == ZNN_RECTIFY) return znn_transfer_bwd(maps, voxels, gy, y, gx, stream);
    if (fn != ZNN_LOGISTIC && fn != ZNN_TANH) return fail(ZNN_EINVAL, "unknown transfer function %d", fn);
    if (maps < 1 || voxels < 1) return fail(ZNN_EINVAL, "maps and voxels must be >= 1");
    if (!gy || !y || !gx) return fail(ZNN_EINVAL, "NULL argument");
    const long total = (long)maps * voxels;
    int rc = check_count(total);
    if (rc != ZNN_OK) return rc;
    const dim3 grid((unsigned)((total + 255) / 256));
    if (fn == ZNN_LOGISTIC)
        ZNN_LAUNCH("transfer backward (logistic)", (hipStream_t)stream, k_transfer_fn_bwd<ZNN_LOGISTIC>, grid, dim3(256), 0,
                   total, gy, y, gx);
    else
        ZNN_LAUNCH("transfer backward (tanh)", (hipStream_t)stream, k_transfer_fn_bwd<ZNN_TANH>, grid, dim3(256), 0,
                   total, gy, y, gx);
    return check_launch("transfer backward");
}

int znn_bias_grad(int32_t maps, int64_t voxels, const float* g, float* gb, void* stream)
{
    if (maps < 1 || voxels < 1) return fail(ZNN_EINVAL, "maps and voxels must be >= 1");
    if (!g || !gb) return fail(ZNN_EINVAL, "NULL argument");
    ZNN_LAUNCH("bias gradient", (hipStream_t)stream, k_bias_grad, dim3((unsigned)maps), dim3(1024), 0, (long)voxels, g, gb);
    return check_launch("bias gradient");
}

int znn_square_loss_grad(int64_t count, const float* out, const float* target, float* g, void* stream)
{
    int rc = check_count(count);
    if (rc != ZNN_OK) return rc;
    if (!out || !target || !g) return fail(ZNN_EINVAL, "NULL argument");
    ZNN_LAUNCH("loss gradient", (hipStream_t)stream, k_sub, dim3((unsigned)((count + 255) / 256)), dim3(256), 0,
                       (long)count, out, target, g);
    return check_launch("loss gradient");
}

int znn_cross_entropy_loss_grad(int64_t count, const float* out, const float* target, float* g, void* stream)
{
    int rc = check_count(count);
    if (rc != ZNN_OK) return rc;
    if (!out || !target || !g) return fail(ZNN_EINVAL, "NULL argument");
    ZNN_LAUNCH("loss gradient (cross-entropy)", (hipStream_t)stream, k_cross_entropy_grad,
               dim3((unsigned)((count + 255) / 256)), dim3(256), 0, (long)count, out, target, g);
    return check_launch("loss gradient");
}

int znn_accumulate(int64_t count, const float* x, float* y, void* stream)
{
    int rc = check_count(count);
    if (rc != ZNN_OK) return rc;
    if (!x || !y) return fail(ZNN_EINVAL, "NULL argument");
    ZNN_LAUNCH("node sum", (hipStream_t)stream, k_accumulate, dim3((unsigned)((count + 255) / 256)), dim3(256), 0,
               (long)count, x, y);
    return check_launch("node sum");
}

int znn_sgd_update(int64_t count, float eta, const float* g, float* p, void* stream)
{
    int rc = check_count(count);
    if (rc != ZNN_OK) return rc;
    if (!g || !p) return fail(ZNN_EINVAL, "NULL argument");
    ZNN_LAUNCH("SGD update", (hipStream_t)stream, k_sgd, dim3((unsigned)((count + 255) / 256)), dim3(256), 0,
                       (long)count, eta, g, p);
    return check_launch("SGD update");
}

}  // extern "C"
