// One-time launch state, kept per device and safe to use from several host threads
// (distinct stage handles may be driven from distinct threads, on distinct devices).
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>

constexpr int EP_MAX_DEVICES = 64;

// Compute units of the current device; asked once per device.
inline hipError_t ep_device_cu_count(int *cus)
{
    static std::atomic<int> cache[EP_MAX_DEVICES];          // zero-initialised
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool cached = dev >= 0 && dev < EP_MAX_DEVICES;
    int n = cached ? cache[dev].load(std::memory_order_acquire) : 0;
    if (n == 0) {
        if ((e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
        if (n < 1) return hipErrorInvalidDevice;
        if (cached) cache[dev].store(n, std::memory_order_release);    // every thread stores the same value
    }
    *cus = n;
    return hipSuccess;
}

// Raises a kernel's dynamic-LDS limit once per device.  One object per kernel instantiation
// (a function-local static of its launcher).  The attribute call is idempotent, so two threads
// that both find the bit clear may both make it; the bit is set only after a successful call.
struct EpSmemLimit {
    std::atomic<uint64_t> done{0};
    hipError_t ensure(const void *kernel, int bytes)
    {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        const bool tracked = dev >= 0 && dev < EP_MAX_DEVICES;
        if (tracked && (done.load(std::memory_order_acquire) >> dev & 1)) return hipSuccess;
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (e == hipSuccess && tracked) done.fetch_or(1ull << dev, std::memory_order_release);
        return e;
    }
};
