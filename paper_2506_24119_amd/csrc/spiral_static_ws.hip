// A decode step that runs on the library's own scratch memory, for callers that cannot allocate device
// memory or pass a workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
// The scratch array is a file-scope device array of a fixed, modest size; each GPU the library runs on holds
// its own copy at its own address until the process ends.  Host code never uses the array's name as an
// address: the device address is looked up once per device and passed to the kernels like any workspace.
#include <cstdio>
#include <mutex>

#include "spiral_internal.h"

namespace {

__device__ __align__(256) unsigned char scratch[SPIRAL_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of the current GPU's copy of `scratch`, looked up on the first call on that device.
int scratch_of_current_device(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return spiral_set_error(SPIRAL_ERR_HIP, hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return spiral_set_error(SPIRAL_ERR_HIP, "decode_step_static: device index out of range");
    std::lock_guard<std::mutex> lock(g_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return spiral_set_error(SPIRAL_ERR_HIP, hipGetErrorString(e));
        if (!ptr) return spiral_set_error(SPIRAL_ERR_HIP, "decode_step_static: no device address for the scratch array");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SPIRAL_OK;
}

}  // namespace

extern "C" size_t spiral_static_workspace_bytes(void) { return SPIRAL_STATIC_WORKSPACE_BYTES; }

extern "C" int spiral_decode_step_static(spiral_model* m, spiral_kv_pool* p, const int32_t* host_seq_ids, int B,
                                         const int32_t* dev_in_tokens, float* dev_logits, void* stream) {
    size_t need = 0;
    int rc = spiral_decode_workspace_need(m, p, host_seq_ids, B, "decode_step_static", &need);
    if (rc) return rc;
    if (need > SPIRAL_STATIC_WORKSPACE_BYTES) {
        char msg[256];
        snprintf(msg, sizeof(msg), "decode_step_static: this step needs %zu bytes of workspace, the built-in scratch holds %zu; "
                 "use spiral_decode_step with a caller-owned workspace", need, (size_t)SPIRAL_STATIC_WORKSPACE_BYTES);
        return spiral_set_error(SPIRAL_ERR_OOM_KV, msg);
    }
    void* ws = nullptr;
    rc = scratch_of_current_device(&ws);
    if (rc) return rc;
    // the step's kernels overwrite every part of the workspace they read, so nothing has to be cleared between calls
    return spiral_decode_on_workspace(m, p, host_seq_ids, B, dev_in_tokens, ws, SPIRAL_STATIC_WORKSPACE_BYTES, dev_logits,
                                              stream, "decode_step_static");
}
