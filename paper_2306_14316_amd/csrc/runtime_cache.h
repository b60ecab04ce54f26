// What the launchers need to know about the device and about their own kernels,
// asked of the HIP runtime once per (device, kernel) and remembered: the number
// of compute units, how many workgroups of a kernel fit on one, and whether the
// kernel's dynamic-LDS limit has been raised yet.  Small layers are bound by the
// host side of a launch, and each of those queries costs as much as the launch.
//
// The tables are written once with the same value by whichever thread gets there
// first and only read afterwards (relaxed atomics), so the library stays
// re-entrant and needs no lock.  Devices with an ordinal of kMaxDevices or more
// are served uncached.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>

namespace im2win {

constexpr int kMaxDevices = 64;

// Current device and its number of compute units.
inline hipError_t device_cus(int *dev, int *ncu)
{
    static std::atomic<int> table[kMaxDevices];   // zero-initialised: 0 = not asked yet
    hipError_t e = hipGetDevice(dev);
    if (e != hipSuccess) return e;
    const bool cached = *dev >= 0 && *dev < kMaxDevices;
    if (cached) {
        const int v = table[*dev].load(std::memory_order_relaxed);
        if (v > 0) { *ncu = v; return hipSuccess; }
    }
    e = hipDeviceGetAttribute(ncu, hipDeviceAttributeMultiprocessorCount, *dev);
    if (e == hipSuccess && cached && *ncu > 0) table[*dev].store(*ncu, std::memory_order_relaxed);
    return e;
}

// One kernel's per-device facts.  A launcher keeps one of these per kernel instance in a
// function-local static.
struct KernelCache {
    std::atomic<int> lds_limit[kMaxDevices];   // dynamic-LDS bytes the kernel has been allowed so far
    std::atomic<int> per_cu[kMaxDevices];      // resident workgroups per compute unit (0 = not asked yet)
};

// Allows `kern` `lds` bytes of dynamic LDS on device `dev` (needed above 48 KiB), once.
inline hipError_t allow_dynamic_lds(KernelCache &kc, const void *kern, size_t lds, int dev)
{
    if (lds <= 48 * 1024) return hipSuccess;
    const bool cached = dev >= 0 && dev < kMaxDevices;
    if (cached && kc.lds_limit[dev].load(std::memory_order_relaxed) >= (int)lds) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess && cached) kc.lds_limit[dev].store((int)lds, std::memory_order_relaxed);
    return e;
}

// Resident workgroups of `kern` per compute unit at this block size and LDS use (fixed per kernel
// instance by its launcher), asked once per device.
inline hipError_t resident_per_cu(KernelCache &kc, const void *kern, int threads, size_t lds, int dev, int *per_cu)
{
    const bool cached = dev >= 0 && dev < kMaxDevices;
    if (cached) {
        const int v = kc.per_cu[dev].load(std::memory_order_relaxed);
        if (v > 0) { *per_cu = v; return hipSuccess; }
    }
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(per_cu, kern, threads, lds);
    if (e == hipSuccess && cached && *per_cu > 0) kc.per_cu[dev].store(*per_cu, std::memory_order_relaxed);
    return e;
}

}  // namespace im2win
