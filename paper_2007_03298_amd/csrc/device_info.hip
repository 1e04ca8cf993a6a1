// Attributes of the current device that the launch rules depend on: the number
// of compute units (how many workgroups fill the chip once) and the LDS per
// compute unit (what an LDS request has to be so that a given number of
// workgroups fit).  Queried once per device and process.
#include <hip/hip_runtime.h>

#include <atomic>

#include "ds_internal.h"

namespace {

constexpr int kMaxDevices = 64;
// compute units in the upper, LDS bytes in the lower 32 bits; 0 = not read yet.
// Two threads that race here both store the same value.
std::atomic<uint64_t> g_cache[kMaxDevices];

}  // namespace

int ds::device_info(DeviceInfo* out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return DS_ERR_HIP;
    const bool cached = dev >= 0 && dev < kMaxDevices;
    uint64_t packed = cached ? g_cache[dev].load(std::memory_order_relaxed) : 0;
    if (packed == 0) {
        int cus = 0, lds = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return DS_ERR_HIP;
        if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) != hipSuccess)
            return DS_ERR_HIP;
        if (cus < 1 || lds < 1) return DS_ERR_HIP;
        packed = (static_cast<uint64_t>(cus) << 32) | static_cast<uint32_t>(lds);
        if (cached) g_cache[dev].store(packed, std::memory_order_relaxed);
    }
    out->compute_units = static_cast<int>(packed >> 32);
    out->lds_per_cu = static_cast<unsigned>(packed & 0xffffffffu);
    return DS_OK;
}
