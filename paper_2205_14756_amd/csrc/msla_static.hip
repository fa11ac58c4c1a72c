// msla_multiscale_state_static: msla_multiscale_state for callers that cannot allocate (code under
// HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  The per-state buffers
// that the other entry point takes from the caller's workspace (per-workgroup partial states, the
// summed states, their MFMA-operand form and scales) live here in a file-scope device array.
//
// Each GPU holds its own copy of the array at its own address until the process ends.  In host code
// the array's name is only a stand-in: the device address is asked for once per device with
// hipGetSymbolAddress and that pointer is what every kernel argument and copy uses.
#include "../../include/msla.h"

#include <hip/hip_runtime.h>

namespace msla {
int multiscale_state_small(const void* qkv, const void* w_dw, const void* w_gpw, void* q_ms, float* kv,
                           void* scratch, size_t scratch_bytes, int B, int H, int W, int heads, int head_dim,
                           const int* scales, int n_scales, int dt, hipStream_t stream);
}

namespace {

constexpr size_t kScratchBytes = MSLA_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};     // device address of `scratch` on each device, once known

// The calling thread's current device's copy of the array (nullptr on failure).
void* scratch_on_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void* p = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (p == nullptr) {
        void* q = nullptr;
        if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || q == nullptr) return nullptr;
        __atomic_store_n(&g_scratch_ptr[dev], q, __ATOMIC_RELEASE);   // two threads racing store the same value
        p = q;
    }
    return p;
}

}  // namespace

extern "C" msla_status msla_multiscale_state_static(const void* qkv, const void* w_dw, const void* w_gpw,
                                                    void* q_ms, float* kv, int B, int H, int W, int heads,
                                                    int head_dim, const int* scales, int n_scales,
                                                    msla_dtype dt, void* stream) {
    if (q_ms == nullptr) return MSLA_ERR_INVALID_ARG;
    void* ptr = scratch_on_current_device();
    if (ptr == nullptr) return MSLA_ERR_LAUNCH;
    // (a shape whose per-state buffers exceed the array comes back as MSLA_ERR_WORKSPACE, before any launch)
    return (msla_status)msla::multiscale_state_small(qkv, w_dw, w_gpw, q_ms, kv, ptr, kScratchBytes, B, H, W, heads,
                                                     head_dim, scales, n_scales, (int)dt,
                                                     static_cast<hipStream_t>(stream));
}
