// Cross-attention for callers that may not allocate device memory: the workspace of
// dit_cross_attn_forward is a device array that is part of the library image instead of a caller's
// buffer.  Everything else -- validation, kernel sequence, kernels -- is dit_cross_attn_forward itself.
#include <mutex>

#include "../../include/dit_attn.h"
#include "dit_attn_internal.h"

// One copy per GPU that loads the library, held until the process ends.  Host code never uses this
// name as an address: it is the handle hipGetSymbolAddress resolves, per device.
static __device__ __align__(256) unsigned char scratch[DIT_STATIC_WORKSPACE_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, once resolved

// Address of the array on the current device; resolved on the first call there and kept.
dit_status scratch_of_current_device(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return static_cast<dit_status>(dit::report_hip_error(e, "hipGetDevice"));
    if (dev < 0 || dev >= kMaxDevices) return DIT_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return static_cast<dit_status>(dit::report_hip_error(e, "hipGetSymbolAddress"));
        if (!p || (reinterpret_cast<uintptr_t>(p) & 255u)) return DIT_ERR_WORKSPACE;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return DIT_OK;
}

}  // namespace

extern "C" dit_status dit_cross_attn_forward_static(const void* q, const void* k, const void* v,
                                                    const uint8_t* kv_valid, void* out, float* lse,
                                                    const dit_cross_attn_params* p, void* stream) {
    if (!p) return DIT_ERR_INVALID_ARG;
    // 0 means the parameters are invalid: let the ordinary entry point name the reason (its checks of
    // the parameters come before any look at the workspace)
    const size_t need = dit_cross_attn_workspace_bytes(p);
    if (need > (size_t)DIT_STATIC_WORKSPACE_BYTES) return DIT_ERR_WORKSPACE;
    void* ws = nullptr;
    if (need > 0) {
        const dit_status st = scratch_of_current_device(&ws);
        if (st != DIT_OK) return st;
    }
    return dit_cross_attn_forward(q, k, v, kv_valid, out, lse, p, ws, ws ? (size_t)DIT_STATIC_WORKSPACE_BYTES : 0,
                                  stream);
}
