// impact_loss_fwd_bwd_static: the loss on a gathered batch with the workspace (per-tile partial sums of the
// loss terms; for small batches also the time segments' scan pairs) in a device array that is part of the
// library's code object, for callers that cannot allocate device memory.
#include <mutex>

#include "impact_internal.h"

namespace {

// One copy per GPU the library runs on, held until the process ends.
static __device__ __align__(256) unsigned char scratch[IMPACT_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
void *g_scratch_ptr[kMaxDevices];      // device address of `scratch` on each device, once looked up

// The array's address on the current device.  In host code the name `scratch` is only a handle for the
// symbol; the memory is reached through the address the runtime reports, which differs from GPU to GPU.
impact_status_t scratch_on_current_device(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return IMPACT_ERR_HIP;
    }
    std::lock_guard<std::mutex> g(g_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return IMPACT_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return IMPACT_OK;
}

}  // namespace

extern "C" impact_status_t impact_loss_fwd_bwd_static(int32_t dist, int32_t batch_dtype, int32_t T, int32_t B, int32_t A,
                                                      const void *learner_dist, const float *values,
                                                      const float *bootstrap, const impact_batch_t *batch,
                                                      const impact_loss_config_t *cfg, const impact_loss_out_t *out,
                                                      impact_stream_t stream)
{
    const size_t need = impact_loss_workspace_bytes(dist, T, B, A);
    if (need == 0) return IMPACT_ERR_INVALID_ARG;
    if (need > (size_t)IMPACT_STATIC_WORKSPACE_BYTES) return IMPACT_ERR_TOO_LARGE;
    void *ws = nullptr;
    const impact_status_t st = scratch_on_current_device(&ws);
    if (st != IMPACT_OK) return st;
    // Nothing in the workspace has to start at zero: every tile stores its partial sums before the
    // reduction launch reads them, and the segmented form writes each pair before the launch that reads it.
    return impact_loss_fwd_bwd(dist, batch_dtype, T, B, A, learner_dist, values, bootstrap, batch, cfg, out, ws,
                               (size_t)IMPACT_STATIC_WORKSPACE_BYTES, stream);
}
