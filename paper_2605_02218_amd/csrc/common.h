// Shared device helpers for the gfx950 kernels (wave64, CDNA4).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace covspec {

typedef unsigned short bf16_t;  // raw bf16 bits
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef double f64x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ float bf16lo_to_f32(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t packed) { return __uint_as_float(packed & 0xFFFF0000u); }

// float -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ bf16_t f32_to_bf16_rne(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
template <typename T>
__device__ __forceinline__ T wave_max(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) { T w = __shfl_xor(v, o, 64); v = w > v ? w : v; }
  return v;
}
template <typename T>
__device__ __forceinline__ T wave_min(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) { T w = __shfl_xor(v, o, 64); v = w < v ? w : v; }
  return v;
}

// fp32 -> uint32 key whose unsigned order equals the float order (-0 is folded onto +0).
__device__ __forceinline__ uint32_t float_order_key(float f) {
  uint32_t u = __float_as_uint(f + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Exclusive prefix sum of one int per thread over a 1024-thread block (blocked order = thread order).
// `wsum` is 17 ints of LDS; the block total is returned in *total.  Contains barriers: call uniformly.
__device__ __forceinline__ int block_exscan_1024(int v, int* wsum, int* total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int t = __shfl_up(inc, o, 64);
    if (lane >= o) inc += t;
  }
  __syncthreads();
  if (lane == 63) wsum[w] = inc;
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int k = 0; k < 16; ++k) { int t = wsum[k]; wsum[k] = run; run += t; }
    wsum[16] = run;
  }
  __syncthreads();
  *total = wsum[16];
  return wsum[w] + inc - v;
}

// Barrier in global memory over the workgroups that work on one image.  `arrived` only grows; `target` is the
// value it reaches when all of them have arrived at this barrier.  Every thread's earlier global writes are
// visible to every thread of the group behind the barrier (device-scope release before, acquire after: the
// XCDs' L2s are not coherent with one another).  The wait is bounded: when it exceeds `limit_ticks` of the
// 100 MHz wall clock, or another workgroup of the image has reported that, `failed` is set and false is
// returned; the caller then gives up on the image.  Call uniformly from all threads; `s_flag` is one int of LDS.
struct ImageBarrier {
  unsigned int arrived;
  int failed;
};
constexpr long long kBarrierLimitTicks = 200000000LL;   // 2 s, the default of `limit_ticks`

__device__ __forceinline__ bool image_barrier_wait(ImageBarrier* bar, unsigned int target, int* s_flag, long long limit_ticks) {
  // Every wave first waits until its own stores have been acknowledged by the L2 (vmcnt counts loads and
  // stores on this architecture); the cache maintenance itself acts on the CU's L1 and the XCD's L2, not on a
  // wave, so one thread issues it for the workgroup: write-back before the arrival, invalidate after the wait.
  __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0)
  __syncthreads();
  if (threadIdx.x == 0) {
    int ok = 1;
    __threadfence();
    __hip_atomic_fetch_add(&bar->arrived, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    const long long t0 = wall_clock64();
    while (__hip_atomic_load(&bar->arrived, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < target) {
      if (__hip_atomic_load(&bar->failed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0 ||
          wall_clock64() - t0 > limit_ticks) {
        ok = 0;
        break;
      }
      __builtin_amdgcn_s_sleep(4);
    }
    if (!ok) __hip_atomic_store(&bar->failed, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __threadfence();
    *s_flag = ok;
  }
  __syncthreads();
  return *s_flag != 0;
}

}  // namespace covspec
