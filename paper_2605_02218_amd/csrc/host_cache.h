// Host-side caches of per-device facts (a kernel's raised dynamic-LDS limit, how many of its workgroups a
// device holds at once).  One slot per device, filled on first use with that device current; readers and
// writers on several host threads are safe (two threads that race compute and store the same value).
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>

namespace covspec {

constexpr int kMaxDevices = 64;

struct PerDeviceInt {
  std::atomic<int> slot[kMaxDevices];   // 0: not computed yet (zero-initialised as a static)

  // *out = the cached value for the current device; `compute(dev, &value)` runs when there is none and must
  // produce a value > 0.
  template <typename F>
  hipError_t get(F compute, int* out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    int v = slot[dev].load(std::memory_order_acquire);
    if (v == 0) {
      if ((e = compute(dev, &v)) != hipSuccess) return e;
      if (v <= 0) return hipErrorInvalidValue;
      slot[dev].store(v, std::memory_order_release);
    }
    *out = v;
    return hipSuccess;
  }
};

// Raises a kernel's dynamic-LDS limit to `bytes` once per device (again when a later call needs more).
inline hipError_t ensure_dynamic_lds(PerDeviceInt& cache, const void* kernel, size_t bytes) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if ((size_t)cache.slot[dev].load(std::memory_order_acquire) >= bytes) return hipSuccess;
  if ((e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes)) != hipSuccess) return e;
  cache.slot[dev].store((int)bytes, std::memory_order_release);
  return hipSuccess;
}

// Workgroups of `kernel` (block size, dynamic LDS) that the current device holds at the same time.
template <typename K>
inline hipError_t resident_workgroups(PerDeviceInt& cache, K kernel, int block, size_t lds, int* out) {
  return cache.get(
      [&](int dev, int* v) -> hipError_t {
        int per_cu = 0, cus = 0;
        hipError_t e;
        if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
        if ((e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, block, lds)) != hipSuccess) return e;
        *v = per_cu * cus;
        return hipSuccess;
      },
      out);
}

}  // namespace covspec
