// Status strings, the per-thread HIP error slot and device queries.
#include "nf4_host.hpp"

namespace nf4 {

thread_local int g_last_hip_error = 0;

int compute_units() {
    thread_local int cached = 0;
    if (cached > 0) return cached;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return 256;  // MI355X; only sizes the grid, never correctness
    cached = cus;
    return cached;
}

}  // namespace nf4

extern "C" int nf4_last_hip_error(void) { return nf4::g_last_hip_error; }

extern "C" const char* nf4_status_string(int status) {
    switch (status) {
        case NF4_OK: return "NF4_OK";
        case NF4_ERR_NULL: return "NF4_ERR_NULL";
        case NF4_ERR_SIZE: return "NF4_ERR_SIZE";
        case NF4_ERR_BLOCKSIZE: return "NF4_ERR_BLOCKSIZE";
        case NF4_ERR_DTYPE: return "NF4_ERR_DTYPE";
        case NF4_ERR_ALIGN: return "NF4_ERR_ALIGN";
        case NF4_ERR_SHAPE: return "NF4_ERR_SHAPE";
        case NF4_ERR_HIP: return "NF4_ERR_HIP";
        default: return "NF4_ERR_UNKNOWN";
    }
}
