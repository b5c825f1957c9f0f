// deltanet_fwd_static: the forward pass for callers that cannot allocate device memory (code under HIP graph capture,
// tight serving loops, harnesses that forbid hipMalloc).  It is deltanet_fwd with the scratch buffer taken from a
// device array that lives in this library's code object instead of from a caller-provided workspace.
#include "../../include/deltanet.h"

#include <hip/hip_runtime.h>

#include <atomic>

namespace {

// The scratch buffer: one copy per GPU, at that GPU's own address, held from the moment the code object is loaded there
// until the process ends.  In host code the name `scratch` is only a handle for hipGetSymbolAddress, never an address.
static __device__ __align__(256) unsigned char scratch[DN_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_of_device[kMaxDevices];

// the current device's copy of the array; asked for once per device, with that device current
int scratch_of_current_device(void **out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DN_ERR_LAUNCH;
    void *ptr = g_scratch_of_device[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return DN_ERR_LAUNCH;
        g_scratch_of_device[dev].store(ptr, std::memory_order_release); // (two threads would store the same address)
    }
    *out = ptr;
    return DN_OK;
}

} // namespace

extern "C" int deltanet_fwd_static(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                                   const float *initial_state, void *o, float *final_state, void *hip_stream) {
    size_t need = 0;
    if (const int rc = deltanet_workspace_bytes(shape, 0, &need)) return rc;
    if (need > (size_t)DN_STATIC_SCRATCH_BYTES) return DN_ERR_WORKSPACE; // the shape needs more scratch than the array holds
    void *ptr = nullptr;
    if (const int rc = scratch_of_current_device(&ptr)) return rc;
    // Nothing in the array has to start at zero: the pass writes every tile of it before reading that tile.
    return deltanet_fwd(shape, q, k, v, beta, initial_state, o, final_state, ptr, (size_t)DN_STATIC_SCRATCH_BYTES, hip_stream);
}
