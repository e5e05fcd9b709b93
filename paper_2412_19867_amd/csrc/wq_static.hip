// wq_conv_forward for callers that cannot allocate device memory: the workspace
// (int8 Winograd-domain activations, their scales, the fp32 scratch of the
// two-kernel variants) lives in a file-scope device array instead of a caller
// buffer.  Every GPU the library runs on holds its own copy of the array at
// its own address; the address is looked up once per device and cached.
#include <mutex>

#include "wq_internal.h"

namespace {

// the library-owned workspace: one per GPU, held until the process ends
static __device__ __align__(256) unsigned char scratch[WQ_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on device d, or nullptr

// Device address of this GPU's copy of `scratch` (the array's name is only a
// host-side stand-in: it must never be handed to a kernel or a memset itself).
hipError_t scratch_address(void **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(g_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // with device `dev` current
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

extern "C" wq_status_t wq_conv_forward_static(const wq_plan_t *plan, void *stream, const float *x_dev,
                                              const void *weight_blob_dev, size_t blob_bytes, float *y_dev) {
    if (!plan || !x_dev || !weight_blob_dev || !y_dev) return WQ_ERR_INVALID_ARG;
    // sizes first, on the host: a plan whose workspace does not fit is refused before any device call
    if (plan->lay.ws_bytes > (uint64_t)WQ_STATIC_WORKSPACE_BYTES) return WQ_ERR_WORKSPACE;
    void *ws = nullptr;
    if (scratch_address(&ws) != hipSuccess) return WQ_ERR_DEVICE;
    // Every byte of the workspace a forward pass reads it has written before in the same pass
    // (codes and scales of all padded rows, then the fp32 scratch), so nothing needs clearing
    // although the array keeps the previous call's contents.
    return wq_conv_forward(plan, stream, x_dev, weight_blob_dev, blob_bytes, ws,
                           (size_t)WQ_STATIC_WORKSPACE_BYTES, y_dev);
}
