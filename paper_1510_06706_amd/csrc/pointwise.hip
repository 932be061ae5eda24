// Max-filtering and its Jacobian, the transfer-function edges, and the small
// elementwise / reduction steps of a training round.
#include "znn_internal.h"

namespace znn {

// Max-filtering (Section 2).  The window is scanned in ascending flat input
// offset with a strict '>' so the smallest offset wins among equal values.
__global__ void __launch_bounds__(256)
k_maxfilter_fwd(int maps, int nz, int ny, int nx, int wz, int wy, int wx,
                const float* __restrict__ in, float* __restrict__ out, int* __restrict__ idx)
{
    const int oz = nz - wz + 1, oy = ny - wy + 1, ox = nx - wx + 1;
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
                const int q = ((z + a) * ny + (y + b)) * nx + (x + c);
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
k_maxfilter_bwd(int maps, int nz, int ny, int nx, int wz, int wy, int wx,
                const float* __restrict__ gout, const int* __restrict__ idx, float* __restrict__ gin)
{
    const int oz = nz - wz + 1, oy = ny - wy + 1, ox = nx - wx + 1;
    const long ovol = (long)oz * oy * ox, nvol = (long)nz * ny * nx;
    const long t = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= nvol * maps) return;
    const int m = (int)(t / nvol);
    const int q = (int)(t % nvol);
    const int x = q % nx, y = (q / nx) % ny, z = q / (nx * ny);
    const int z0 = max(z - wz + 1, 0), z1 = min(z, oz - 1);
    const int y0 = max(y - wy + 1, 0), y1 = min(y, oy - 1);
    const int x0 = max(x - wx + 1, 0), x1 = min(x, ox - 1);
    const float* g = gout + m * ovol;
    const int* id = idx + m * ovol;
    float acc = 0.f;
    for (int pz = z0; pz <= z1; ++pz)
        for (int py = y0; py <= y1; ++py)
            for (int px = x0; px <= x1; ++px) {
                const long p = ((long)pz * oy + py) * ox + px;
                if (id[p] == q) acc += g[p];
            }
    gin[t] = acc;
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

// One block per map; every thread sums a fixed strided subset, then a fixed tree.
__global__ void __launch_bounds__(256)
k_bias_grad(long voxels, const float* __restrict__ g, float* __restrict__ gb)
{
    __shared__ float red[256];
    const float* p = g + (long)blockIdx.x * voxels;
    float acc = 0.f;
    for (long t = threadIdx.x; t < voxels; t += 256) acc += p[t];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
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

static int check_filter(int32_t maps, znn_vec3 n, znn_vec3 win)
{
    if (maps < 1) return fail(ZNN_EINVAL, "maps must be >= 1");
    const int nn[3] = {n.z, n.y, n.x}, ww[3] = {win.z, win.y, win.x};
    for (int a = 0; a < 3; ++a) {
        if (nn[a] < 1 || ww[a] < 1) return fail(ZNN_EINVAL, "image and window extents must be >= 1");
        if (ww[a] > nn[a]) return fail(ZNN_EINVAL, "window extent %d exceeds image extent %d on axis %d", ww[a], nn[a], a);
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

int znn_maxfilter3d_fwd(int32_t maps, znn_vec3 n, znn_vec3 win, const float* in,
                        float* out, int32_t* idx, void* stream)
{
    int rc = check_filter(maps, n, win);
    if (rc != ZNN_OK) return rc;
    if (!in || !out || !idx) return fail(ZNN_EINVAL, "NULL argument");
    const long total = (long)maps * (n.z - win.z + 1) * (n.y - win.y + 1) * (n.x - win.x + 1);
    ZNN_LAUNCH("max-filter forward", (hipStream_t)stream, k_maxfilter_fwd, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       maps, n.z, n.y, n.x, win.z, win.y, win.x, in, out, idx);
    return check_launch("max-filter forward");
}

int znn_maxfilter3d_bwd(int32_t maps, znn_vec3 n, znn_vec3 win, const float* gout,
                        const int32_t* idx, float* gin, void* stream)
{
    int rc = check_filter(maps, n, win);
    if (rc != ZNN_OK) return rc;
    if (!gout || !idx || !gin) return fail(ZNN_EINVAL, "NULL argument");
    const long total = (long)maps * n.z * n.y * n.x;
    ZNN_LAUNCH("max-filter backward", (hipStream_t)stream, k_maxfilter_bwd, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       maps, n.z, n.y, n.x, win.z, win.y, win.x, gout, idx, gin);
    return check_launch("max-filter backward");
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

int znn_bias_grad(int32_t maps, int64_t voxels, const float* g, float* gb, void* stream)
{
    if (maps < 1 || voxels < 1) return fail(ZNN_EINVAL, "maps and voxels must be >= 1");
    if (!g || !gb) return fail(ZNN_EINVAL, "NULL argument");
    ZNN_LAUNCH("bias gradient", (hipStream_t)stream, k_bias_grad, dim3((unsigned)maps), dim3(256), 0, (long)voxels, g, gb);
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
