// Library-wide state: error record, device properties, version.
#include <hip/hip_runtime.h>

#include <atomic>

#include "rov_internal.h"

namespace rov {

namespace {
thread_local int t_last_hip_error = 0;
std::atomic<int> g_cu_count{0};
}  // namespace

int record_hip_error(hipError_t e) {
    t_last_hip_error = (int)e;
    return ROV_ERR_HIP;
}

int device_cu_count() {
    int n = g_cu_count.load();
    if (n > 0) return n;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess ||
        prop.multiProcessorCount <= 0) {
        n = 256;   // MI355X
    } else {
        n = prop.multiProcessorCount;
    }
    g_cu_count.store(n);
    return n;
}

}  // namespace rov

extern "C" {

int rov_last_hip_error(void) { return rov::t_last_hip_error; }

const char* rov_version(void) { return "rov 0.1 (gfx950)"; }

}  // extern "C"
