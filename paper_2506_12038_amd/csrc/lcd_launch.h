// Host-side helpers of the launchers in the .hip files: per-device bookkeeping.
#pragma once
#include <hip/hip_runtime.h>
#include <atomic>

namespace lcd {

constexpr int kMaxDevices = 64;

// Index of the current device, or -1 (no device, or an index beyond kMaxDevices).
inline int current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return -1;
    return dev;
}

// "This kernel's dynamic-LDS limit has been raised on this device": one flag per device and kernel variant.
// The flags are atomics and raising the limit twice is harmless, so concurrent first calls are safe.
template <int VARIANTS>
struct PerDeviceFlags {
    std::atomic<bool> set[kMaxDevices][VARIANTS] = {};
};

template <int VARIANTS>
inline hipError_t raise_lds_limit_once(PerDeviceFlags<VARIANTS> &flags, int variant, const void *fn, size_t lds_bytes)
{
    const int dev = current_device();
    if (dev < 0) return hipErrorInvalidDevice;
    if (flags.set[dev][variant].load(std::memory_order_acquire)) return hipSuccess;
    if (hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes)) return e;
    flags.set[dev][variant].store(true, std::memory_order_release);
    return hipSuccess;
}

}  // namespace lcd
