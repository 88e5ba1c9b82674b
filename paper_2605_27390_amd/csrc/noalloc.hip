// evospec_active_lmhead_topk_static: the restricted head for callers that cannot allocate device
// memory (code under HIP graph capture, serving loops, harnesses that forbid hipMalloc).  The
// per-slab partial results that the other entry points keep in a caller workspace live here in a
// fixed device array of the library, one copy per GPU.
#include <hip/hip_runtime.h>

#include <mutex>

#include "evospec.h"
#include "launch.hpp"

namespace {

// The scratch itself.  In host code this name is only a handle for hipGetSymbolAddress; the
// device address of each GPU's copy is looked up once per device and kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char g_head_scratch[EVOSPEC_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Device address of the current device's copy of the scratch array (looked up on the first call
// on that device, with that device current).
int scratch_for_current_device(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return evospec::record_hip_error(e);
    if (dev < 0 || dev >= kMaxDevices) return evospec::record_hip_error(hipErrorInvalidDevice);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_head_scratch));
        if (e != hipSuccess) return evospec::record_hip_error(e);
        if (!p) return evospec::record_hip_error(hipErrorInvalidSymbol);
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return EVOSPEC_OK;
}

}  // namespace

extern "C" int evospec_active_lmhead_topk_static(const void* h, int M, int d, const void* W_act,
                                                 const int32_t* ids, int V_act, int layout, int k,
                                                 float* out_vals, int32_t* out_ids, float* out_logz,
                                                 void* stream) {
    // shape errors first, with the same codes as the workspace variant
    size_t need = 0;
    int rc = evospec_workspace_bytes(M, V_act, d, k, &need);
    if (rc) return rc;
    if (need > (size_t)EVOSPEC_STATIC_SCRATCH_BYTES) return EVOSPEC_STATIC_SCRATCH_EXCEEDED;
    if (M == 0) return EVOSPEC_OK;
    void* scratch = nullptr;
    rc = scratch_for_current_device(&scratch);
    if (rc) return rc;
    // Nothing in the scratch has to start at a given value: every slot that the merge reads was
    // written by the slab launch of the same call.
    return evospec::head_impl(h, M, d, W_act, ids, V_act, layout, k, out_vals, out_ids, out_logz, scratch,
                              (size_t)EVOSPEC_STATIC_SCRATCH_BYTES, stream, nullptr);
}
