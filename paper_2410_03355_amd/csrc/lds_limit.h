// Dynamic LDS beyond 64 KiB has to be allowed per kernel and device before the launch.
#pragma once

#include <hip/hip_runtime.h>

#include <map>
#include <mutex>
#include <utility>

namespace lantern {

// Raises the kernel's dynamic-LDS limit to `lds` bytes on the current device unless a limit at
// least as large is already in place: after the first launch of a shape, further launches of it
// (also those recorded into a HIP graph) make no runtime call besides the launch itself.
template <typename K>
inline hipError_t allow_lds(K kernel, size_t lds) {
    if (lds <= 64 * 1024) return hipSuccess;
    static std::mutex mu;
    static std::map<std::pair<const void*, int>, size_t> granted;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const std::pair<const void*, int> key(reinterpret_cast<const void*>(kernel), dev);
    std::lock_guard<std::mutex> lock(mu);
    const auto it = granted.find(key);
    if (it != granted.end() && it->second >= lds) return hipSuccess;
    e = hipFuncSetAttribute(key.first, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess) granted[key] = lds;
    return e;
}

}  // namespace lantern
