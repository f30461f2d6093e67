// Per-device host-side caches: the number of compute units and the "dynamic LDS limit raised" marks, so that a
// launch costs no runtime query after the first one on a device.
#include "hk_internal.h"

namespace hk {
namespace {

constexpr int kMaxDevices = 64;
std::atomic<int> g_cus[kMaxDevices];       // 0: not asked yet

}  // namespace

hipError_t current_device_cus(int *dev, int *cus)
{
    hipError_t e = hipGetDevice(dev);
    if (e != hipSuccess) return e;
    if (*dev < 0 || *dev >= kMaxDevices) return hipErrorInvalidDevice;
    int n = g_cus[*dev].load(std::memory_order_relaxed);
    if (n == 0) {
        e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, *dev);
        if (e != hipSuccess) return e;
        if (n <= 0) return hipErrorInvalidValue;
        g_cus[*dev].store(n, std::memory_order_relaxed);
    }
    *cus = n;
    return hipSuccess;
}

hipError_t allow_dynamic_lds(const void *kernel, int bytes, LdsOnce &once)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    const uint64_t bit = 1ull << dev;
    if (once.done.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) once.done.fetch_or(bit, std::memory_order_release);
    return e;
}

}  // namespace hk
