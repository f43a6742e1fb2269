// vscan_llm_prune_static: stage 2 for callers that may not allocate device memory.
//
// The scratch vscan_llm_prune takes through its `workspace` argument (the per-kv-head partial
// scores between the scoring and the selection kernel) lives here in a file-scope device array.
// In host code the array's NAME is only a stand-in for the symbol: the device address is asked
// for once per device with hipGetSymbolAddress and that pointer - never the name - is what the
// kernels receive.  Every GPU holds its own copy of the array at its own address.
#include <hip/hip_runtime.h>

#include <mutex>

#include "../../include/vscan.h"
#include "log.hpp"

namespace vscan {
int llm_prune_validate(const vscan_llm_desc *d, const void *q, const void *k, const void *v,
                       const void *hidden, const int32_t *kept_idx, const void *k_out,
                       const void *v_out, const void *hidden_out, const float *scores_out,
                       size_t *workspace_bytes);  // api.cpp
}

namespace {

// 16 MiB: the partial scores of 32 sequences x 32 kv heads x 2880 visual tokens take 11.25 MiB.
static __device__ __align__(256) unsigned char scratch[VSCAN_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, once known

// Device address of the scratch array on the current device (NULL on failure).
void *scratch_on_current_device() {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        vscan::logf("static scratch: hipGetDevice -> %s, device %d", hipGetErrorString(e), dev);
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            vscan::logf("static scratch: hipGetSymbolAddress -> %s", hipGetErrorString(e));
            return nullptr;
        }
        vscan::logf("static scratch: device %d holds the array at %p", dev, p);
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

extern "C" int vscan_llm_prune_static(const vscan_llm_desc *desc, const void *q, void *k, void *v,
                                      void *hidden, int32_t *kept_idx, void *k_out, void *v_out,
                                      void *hidden_out, float *scores_out, void *stream) {
    const int status = [&]() -> int {
        // descriptor and pointers first (host only): errors read the same with or without a GPU
        size_t need = 0;
        const int rc = vscan::llm_prune_validate(desc, q, k, v, hidden, kept_idx, k_out, v_out,
                                                 hidden_out, scores_out, &need);
        if (rc != VSCAN_OK) return rc;
        if (need > (size_t)VSCAN_STATIC_SCRATCH_BYTES) return VSCAN_ERR_WORKSPACE;
        if (desc->batch == 0) return VSCAN_OK;  // nothing to enqueue: the GPU is never touched
        void *ws = scratch_on_current_device();
        if (!ws) return VSCAN_ERR_HIP;
        // Every word of the scratch the selection reads has been written by the scoring kernel
        // of the same call, so nothing needs clearing between calls.
        return vscan_llm_prune(desc, q, k, v, hidden, kept_idx, k_out, v_out, hidden_out,
                               scores_out, ws, (size_t)VSCAN_STATIC_SCRATCH_BYTES, stream);
    }();
    if (status != VSCAN_OK)
        vscan::logf("vscan_llm_prune_static -> %d (%s)", status, vscan_status_string(status));
    return status;
}
