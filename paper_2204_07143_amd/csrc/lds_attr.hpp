// Host side: a kernel that asks for more than 64 KB of dynamic LDS needs
// hipFuncAttributeMaxDynamicSharedMemorySize first, per kernel and per device.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace na2d {

// One per kernel instantiation (a function-local static of its launcher): bit d is set once the attribute
// has been set on device d.  Safe to use from several host threads; devices past 63 set it on every launch.
struct LdsAllowed {
    std::atomic<uint64_t> devices{0};
};

template <typename Kern>
inline hipError_t allow_lds(Kern kern, int max_bytes, LdsAllowed &done) {
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    const bool tracked = dev >= 0 && dev < 64;
    const uint64_t bit = tracked ? 1ull << dev : 0ull;
    if (tracked && (done.devices.load(std::memory_order_acquire) & bit)) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, max_bytes);
    if (e == hipSuccess && tracked) done.devices.fetch_or(bit, std::memory_order_release);
    return e;
}

}  // namespace na2d
