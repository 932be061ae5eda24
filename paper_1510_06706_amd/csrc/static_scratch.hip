// Forward pass for callers that cannot allocate device memory (code under HIP graph capture,
// tight serving loops, harnesses that forbid hipMalloc): the scratch that znn_conv3d_fwd takes
// from the caller's workspace (packed weights and partial sums of the direct method; node and
// kernel spectra of the FFT method) lives in a file-scope device array instead.
//
// Every GPU the library runs on holds its own copy of the array, at its own address, until
// the process ends.  The array's name is only a host-side handle: the device address is looked
// up once per device with hipGetSymbolAddress and that address is what the kernels receive.
// All calls on one GPU share the array, so calls that overlap in time on one GPU race.
// Nothing in it has to start at zero: the packer, the transforms and the partial-sum kernels
// write every word they later read.
#include <mutex>

#include "znn_internal.h"

namespace {

constexpr size_t kScratchBytes = ZNN_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device; looked up on the first call per device.
int scratch_of_current_device(void** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return znn::fail(ZNN_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return znn::fail(ZNN_EUNSUPPORTED, "device ordinal %d is out of range", dev);
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return znn::fail(ZNN_EHIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return ZNN_OK;
}

}  // namespace

extern "C" int znn_conv3d_fwd_static(znn_plan* plan, const float* in, const float* w, float* out, void* stream)
{
    if (!plan || !in || !out) return znn::fail(ZNN_EINVAL, "NULL argument");
    size_t need = 0;
    int rc = znn_plan_workspace_bytes(plan, ZNN_PASS_FWD, &need);
    if (rc != ZNN_OK) return rc;
    if (need > kScratchBytes)
        return znn::fail(ZNN_EWORKSPACE, "this layer's forward pass needs %zu bytes of scratch, the built-in array holds %zu; "
                                         "use znn_conv3d_fwd with a workspace", need, kScratchBytes);
    void* ptr = nullptr;
    if ((rc = scratch_of_current_device(&ptr)) != ZNN_OK) return rc;
    return znn_conv3d_fwd(plan, in, w, out, ptr, kScratchBytes, stream);
}
