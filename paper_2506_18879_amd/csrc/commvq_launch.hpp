// Launch helper shared by every translation unit of libcommvq.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>

namespace {

// Raises a kernel's dynamic-LDS limit once per device.  `done` is the call site's own mask (one bit per device
// ordinal); setting the attribute twice is harmless, so two threads racing here only repeat the call.
template <typename Kernel>
inline hipError_t allow_dynamic_lds(Kernel *kernel, int bytes, std::atomic<uint64_t> &done)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
    return e;
}

}  // namespace
