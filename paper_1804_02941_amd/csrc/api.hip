// Status text, error bookkeeping and the one-time device set-up of the C ABI.
#include "dab_internal.h"

#include <atomic>
#include <mutex>

namespace dab {

thread_local int g_last_hip_error = 0;

static std::atomic<int> g_ready[kMaxDevices];
static std::mutex g_setup_lock;

// Set-up of the current device, done once per device: kernels that take more dynamic LDS than a
// launch is granted by default get their limit raised, and the address of the library's own
// device memory is looked up.  Every entry point that depends on it calls this first; after the
// first call on a device it is one hipGetDevice and one atomic load.
int ensure_device_ready(int* dev_out) {
    int dev = 0;
    const hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_failed(e);
    if (dev < 0 || dev >= kMaxDevices) return DAB_ERR_UNSUPPORTED;
    if (dev_out) *dev_out = dev;
    if (g_ready[dev].load(std::memory_order_acquire)) return DAB_OK;
    std::lock_guard<std::mutex> guard(g_setup_lock);
    if (g_ready[dev].load(std::memory_order_relaxed)) return DAB_OK;
    if (int rc = init_binconv()) return rc;
    if (int rc = init_direct()) return rc;
    if (int rc = init_pack()) return rc;
    if (int rc = init_estimate(dev)) return rc;
    g_ready[dev].store(1, std::memory_order_release);
    return DAB_OK;
}

}  // namespace dab

extern "C" {

const char* dab_strerror(int status) {
    switch (status) {
        case DAB_OK: return "ok";
        case DAB_ERR_NULL: return "a required pointer is NULL";
        case DAB_ERR_SHAPE: return "invalid size (non-positive dimension, n < 2 or empty output)";
        case DAB_ERR_ALIGN: return "a buffer is not aligned as the header requires";
        case DAB_ERR_WORKSPACE: return "workspace missing or too small";
        case DAB_ERR_UNSUPPORTED: return "valid problem outside what the kernels cover";
        case DAB_ERR_HIP: return "a HIP call failed (see dab_last_hip_error)";
        default: return "unknown status";
    }
}

int dab_last_hip_error(void) { return dab::g_last_hip_error; }

int dab_init(void) { return dab::ensure_device_ready(nullptr); }

}  // extern "C"
