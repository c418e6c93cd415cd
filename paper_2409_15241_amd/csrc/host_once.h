// Host-side helper of the launchers: raising a kernel's dynamic LDS limit has to happen once per kernel and
// device, and launchers can be entered from several host threads at once (the single-kernel entry points
// take no library lock).
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>
#include <mutex>

struct LdsLimitOnce {
  std::atomic<uint64_t> done{0};     // bit d: the limit is set on device d
  std::mutex m;
  hipError_t ensure(const void* kern, int bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    std::lock_guard<std::mutex> lock(m);
    if (done.load(std::memory_order_relaxed) & bit) return hipSuccess;
    e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
    return e;
  }
};
