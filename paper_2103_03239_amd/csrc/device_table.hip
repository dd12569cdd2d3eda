// Per-device launch facts shared by the kernel translation units: which kernels
// already had their dynamic-LDS limit raised on which device, and the number of
// compute units of each device.  One table per process, guarded by a mutex, filled
// on first use with the device that is current in the calling thread.
#include <mutex>
#include <unordered_map>

#include "moshpit_internal.h"

namespace moshpit {
namespace {

constexpr int kMaxDevices = 64;

struct DeviceFacts {
    int compute_units = 0;                              // 0 = not looked up yet
    std::unordered_map<const void *, int> lds_limit;    // kernel -> bytes already allowed
};

std::mutex g_mutex;
DeviceFacts g_devices[kMaxDevices];

hipError_t current_slot(int *dev)
{
    hipError_t e = hipGetDevice(dev);
    if (e != hipSuccess) return e;
    return (*dev >= 0 && *dev < kMaxDevices) ? hipSuccess : hipErrorInvalidDevice;
}

}  // namespace

hipError_t ensure_dynamic_lds(const void *kernel, int bytes)
{
    int dev = 0;
    hipError_t e = current_slot(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(g_mutex);
    auto &limit = g_devices[dev].lds_limit;
    const auto it = limit.find(kernel);
    if (it != limit.end() && it->second >= bytes) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    limit[kernel] = bytes;
    return hipSuccess;
}

hipError_t current_compute_units(int *out)
{
    int dev = 0;
    hipError_t e = current_slot(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceFacts &f = g_devices[dev];
    if (f.compute_units == 0) {
        int cu = 0;
        e = hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        f.compute_units = cu > 0 ? cu : 256;
    }
    *out = f.compute_units;
    return hipSuccess;
}

}  // namespace moshpit
