// Status text and error bookkeeping of the C ABI.
#include "dab_internal.h"

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

}  // extern "C"
