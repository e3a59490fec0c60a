// Host-side helper: kernels that need more than 48 KB of dynamic LDS must be told so once per
// device (hipFuncSetAttribute); doing it on every launch costs a few microseconds of host time
// that small workloads notice.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>

namespace vitq {

// `done` is one bit per device ordinal (up to 64), owned by the call site (one per kernel).
inline hipError_t allow_dynamic_lds(const void *kernel, size_t bytes, std::atomic<uint64_t> &done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = (dev >= 0 && dev < 64) ? (uint64_t(1) << dev) : 0;
    if (bit && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess && bit) done.fetch_or(bit, std::memory_order_release);
    return e;
}

}  // namespace vitq
