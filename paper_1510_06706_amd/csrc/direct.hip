// Direct method: dispatch between the tiled MFMA kernels and the generic ones.
#include "znn_internal.h"

namespace znn {

int direct_fwd_generic(const Geom& g, const float* in, const float* w, float* out, hipStream_t s);
int direct_bwd_generic(const Geom& g, const float* gout, const float* w, float* gin, hipStream_t s);
int direct_wgrad_generic(const Geom& g, const float* in, const float* gout, float* gw, hipStream_t s);

bool   mfma_conv_supported(const Geom& g, bool backward);
size_t mfma_conv_workspace(const Geom& g, bool backward);
int    mfma_conv(const Geom& g, bool backward, const float* src, const float* w, float* dst, void* ws,
                 hipStream_t s);

bool   mfma_wgrad_supported(const Geom& g);
size_t mfma_wgrad_workspace(const Geom& g);
int    mfma_wgrad(const Geom& g, const float* in, const float* gout, float* gw, void* ws, hipStream_t s);

size_t direct_workspace_bytes(const Geom& g, int pass)
{
    if (pass == ZNN_PASS_FWD) return mfma_conv_workspace(g, false);
    if (pass == ZNN_PASS_BWD) return mfma_conv_workspace(g, true);
    return mfma_wgrad_workspace(g);
}

int direct_fwd(const Geom& g, const float* in, const float* w, float* out, void* ws, hipStream_t s)
{
    if (mfma_conv_supported(g, false)) return mfma_conv(g, false, in, w, out, ws, s);
    return direct_fwd_generic(g, in, w, out, s);
}

int direct_bwd(const Geom& g, const float* gout, const float* w, float* gin, void* ws, hipStream_t s)
{
    if (mfma_conv_supported(g, true)) return mfma_conv(g, true, gout, w, gin, ws, s);
    return direct_bwd_generic(g, gout, w, gin, s);
}

int direct_wgrad(const Geom& g, const float* in, const float* gout, float* gw, void* ws, hipStream_t s)
{
    if (mfma_wgrad_supported(g)) return mfma_wgrad(g, in, gout, gw, ws, s);
    return direct_wgrad_generic(g, in, gout, gw, s);
}

}  // namespace znn
