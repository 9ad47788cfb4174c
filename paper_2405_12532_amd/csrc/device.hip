// Per-device facts the launchers need (compute units, XCDs) and the once-per-device setting of a
// kernel's dynamic LDS limit.  Both are cached per device id behind atomics: the entry points may be
// called from several host threads and on several devices of one process.
#include <atomic>

#include "pyr_internal.h"

namespace pyr {
namespace {

constexpr int kMaxDevices = 64;
std::atomic<int> g_cus[kMaxDevices];      // 0: not queried yet
std::atomic<int> g_xccs[kMaxDevices];

}  // namespace

int device_info(DeviceInfo* out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PYR_ERR_LAUNCH;
    int cus = g_cus[dev].load(std::memory_order_acquire);
    int xccs = g_xccs[dev].load(std::memory_order_acquire);
    if (cus == 0 || xccs == 0) {
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            return PYR_ERR_LAUNCH;
        if (hipDeviceGetAttribute(&xccs, hipDeviceAttributeNumberOfXccs, dev) != hipSuccess || xccs <= 0)
            return PYR_ERR_LAUNCH;
        g_xccs[dev].store(xccs, std::memory_order_release);
        g_cus[dev].store(cus, std::memory_order_release);
    }
    out->device = dev;
    out->compute_units = cus;
    out->xccs = xccs;
    return PYR_OK;
}

int ensure_dynamic_lds(const void* kernel, int bytes, std::atomic<uint64_t>* done_mask) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PYR_ERR_LAUNCH;
    const uint64_t bit = 1ull << dev;
    if (done_mask->load(std::memory_order_acquire) & bit) return PYR_OK;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
        return PYR_ERR_LAUNCH;
    done_mask->fetch_or(bit, std::memory_order_release);     // (two threads may both make the call: it is idempotent)
    return PYR_OK;
}

}  // namespace pyr
