// Library-wide state: error record, device properties, version.
#include <hip/hip_runtime.h>

#include <atomic>
#include <mutex>
#include <utility>
#include <vector>

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

// hipFuncAttributeMaxDynamicSharedMemorySize is a property of (device, kernel): set it the first
// time a kernel is launched on a device and never again (the launch paths call this every time).
int set_max_dynamic_lds(const void* kern, int bytes) {
    static std::mutex mu;
    static std::vector<std::pair<int, const void*>> done;
    int dev = 0;
    ROV_HIP_TRY(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(mu);
    for (const auto& d : done)
        if (d.first == dev && d.second == kern) return ROV_OK;
    ROV_HIP_TRY(hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    done.emplace_back(dev, kern);
    return ROV_OK;
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

// ---- kernel tracing: timing events around the launches made by the schedules
namespace {
struct TraceRec {
    int kind;
    hipEvent_t a, b;
};
std::mutex g_trace_mu;
std::vector<TraceRec> g_trace_pool;     // events are created once and reused
size_t g_trace_used = 0;
std::atomic<int> g_trace_on{0};
constexpr size_t kTraceMax = 16384;
}  // namespace

int trace_begin(int kind, hipStream_t st) {
    const int sel = g_trace_on.load();
    if (sel == 0 || (sel > 0 && !((sel >> kind) & 1))) return -1;
    std::lock_guard<std::mutex> lock(g_trace_mu);
    if (g_trace_used >= kTraceMax) return -1;
    if (g_trace_used == g_trace_pool.size()) {
        TraceRec r{kind, nullptr, nullptr};
        if (hipEventCreate(&r.a) != hipSuccess) return -1;
        if (hipEventCreate(&r.b) != hipSuccess) { (void)hipEventDestroy(r.a); return -1; }
        g_trace_pool.push_back(r);
    }
    const int slot = (int)g_trace_used++;
    g_trace_pool[slot].kind = kind;
    (void)hipEventRecord(g_trace_pool[slot].a, st);
    return slot;
}

void trace_end(int slot, hipStream_t st) {
    if (slot < 0) return;
    std::lock_guard<std::mutex> lock(g_trace_mu);
    (void)hipEventRecord(g_trace_pool[slot].b, st);
}

}  // namespace rov

extern "C" {

int rov_trace_enable(int on) { return rov::g_trace_on.exchange(on); }

int rov_trace_read(int* kinds, float* ms, int max_records, int* n_records) {
    if (n_records == nullptr || max_records < 0 || (max_records > 0 && (kinds == nullptr || ms == nullptr)))
        return ROV_ERR_INVALID;
    std::lock_guard<std::mutex> lock(rov::g_trace_mu);
    int n = 0;
    for (size_t i = 0; i < rov::g_trace_used; ++i) {
        const rov::TraceRec& r = rov::g_trace_pool[i];
        ROV_HIP_TRY(hipEventSynchronize(r.b));
        float t = 0.0f;
        ROV_HIP_TRY(hipEventElapsedTime(&t, r.a, r.b));
        if (n < max_records) {
            kinds[n] = r.kind;
            ms[n] = t;
            ++n;
        }
    }
    rov::g_trace_used = 0;
    *n_records = n;
    return ROV_OK;
}

int rov_last_hip_error(void) { return rov::t_last_hip_error; }

const char* rov_version(void) { return "rov 0.1 (gfx950)"; }

}  // extern "C"
