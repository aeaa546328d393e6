// Once-per-device bookkeeping shared by the kernel launchers of this library.
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>

// Which devices have had a kernel's dynamic-LDS attribute set, and the number of compute units of each (queried
// once).  One object per kernel instantiation (a function-local static).  Thread safe: a race at most repeats
// an idempotent runtime call.
struct PerDeviceOnce {
    static constexpr int MAX_DEV = 64;
    std::atomic<unsigned long long> attr_done{0};
    std::atomic<int> cus[MAX_DEV] = {};

    // Sets hipFuncAttributeMaxDynamicSharedMemorySize for `kern` on the current device unless already done there.
    // Returns the current device, or -1 when the runtime refuses.
    int prepare(const void* kern, int smem) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEV) return -1;
        if (!((attr_done.load(std::memory_order_acquire) >> dev) & 1ull)) {
            if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess) return -1;
            attr_done.fetch_or(1ull << dev, std::memory_order_release);
        }
        return dev;
    }
    // Compute units of device `dev` (0 when the runtime refuses).
    int compute_units(int dev) {
        int n = cus[dev].load(std::memory_order_relaxed);
        if (n == 0) {
            if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
            cus[dev].store(n, std::memory_order_relaxed);
        }
        return n;
    }
};
