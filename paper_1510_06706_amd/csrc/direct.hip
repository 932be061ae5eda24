// Direct method: dispatch between the tiled MFMA kernels and the generic ones.
#include "znn_internal.h"

namespace znn {

int direct_fwd_generic(const Geom& g, const float* in, const float* w, float* out, hipStream_t s);
int direct_bwd_generic(const Geom& g, const float* gout, const float* w, float* gin, hipStream_t s);
int direct_wgrad_generic(const Geom& g, const float* in, const float* gout, float* gw, hipStream_t s);

size_t direct_workspace_bytes(const Geom& g, int pass)
{
    (void)g; (void)pass;
    return 0;
}

int direct_fwd(const Geom& g, const float* in, const float* w, float* out, void* ws, hipStream_t s)
{
    (void)ws;
    return direct_fwd_generic(g, in, w, out, s);
}

int direct_bwd(const Geom& g, const float* gout, const float* w, float* gin, void* ws, hipStream_t s)
{
    (void)ws;
    return direct_bwd_generic(g, gout, w, gin, s);
}

int direct_wgrad(const Geom& g, const float* in, const float* gout, float* gw, void* ws, hipStream_t s)
{
    (void)ws;
    return direct_wgrad_generic(g, in, gout, gw, s);
}

}  // namespace znn
