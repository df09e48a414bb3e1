// Dynamic LDS beyond 64 KiB has to be allowed per kernel and device before the launch.
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <mutex>

namespace lantern {

// Raises the kernel's dynamic-LDS limit to `lds` bytes on the current device unless a limit at
// least as large is already in place.  The steady state is one relaxed atomic load per call: the
// runtime is called (under a lock) only the first time a kernel needs more than it was granted on
// a device, which lantern_prepare does ahead of time for callers that capture HIP graphs.
template <auto Kernel>
inline hipError_t allow_lds(size_t lds) {
    if (lds <= 64 * 1024) return hipSuccess;
    constexpr int MAX_DEVICES = 64;
    static std::atomic<size_t> granted[MAX_DEVICES];   // zero-initialised
    static std::mutex mu;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool tracked = dev >= 0 && dev < MAX_DEVICES;
    if (tracked && granted[dev].load(std::memory_order_acquire) >= lds) return hipSuccess;
    std::lock_guard<std::mutex> lock(mu);
    if (tracked && granted[dev].load(std::memory_order_relaxed) >= lds) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds);
    if (e == hipSuccess && tracked) granted[dev].store(lds, std::memory_order_release);
    return e;
}

}  // namespace lantern
