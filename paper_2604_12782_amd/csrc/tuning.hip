// Process-wide kernel-choice overrides (include/osc_tuning.h) and small per-device caches that keep
// repeated host work (device queries, function attributes) off the launch path.
#include <atomic>

#include "osc_internal.h"
#include "../../include/osc_tuning.h"

namespace osc {

static std::atomic<int> g_knob[TUNE_COUNT] = {{-1}, {-1}, {-1}, {-1}, {-1}};

int tuning(int knob) { return g_knob[knob].load(std::memory_order_relaxed); }

int cu_count() {
    static std::atomic<int> cached[MAX_DEVICES];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return -1;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n > 0) return n;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return -1;
    cached[dev].store(n, std::memory_order_relaxed);
    return n;
}

int reserve_lds(const void* kernel, size_t bytes, unsigned char (&done)[MAX_DEVICES], size_t (&reserved)[MAX_DEVICES]) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES)
        return fail(OSC_ERR_HIP, "cannot read the current device");
    // racing first calls from two threads both set the attribute to the value they need; harmless
    if (done[dev] && reserved[dev] >= bytes) return OSC_OK;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) {
        (void)hipGetLastError();
        return fail(OSC_ERR_HIP, "cannot reserve %zu bytes of LDS", bytes);
    }
    reserved[dev] = bytes;
    done[dev] = 1;
    return OSC_OK;
}

}  // namespace osc

extern "C" int osc_tuning_set(int knob, int value) {
    if (knob < 0 || knob >= osc::TUNE_COUNT) return osc::fail(OSC_ERR_UNSUPPORTED, "osc_tuning_set: knob %d", knob);
    osc::g_knob[knob].store(value < 0 ? -1 : value, std::memory_order_relaxed);
    return OSC_OK;
}

extern "C" int osc_tuning_get(int knob) {
    if (knob < 0 || knob >= osc::TUNE_COUNT) return -1;
    return osc::tuning(knob);
}
