// Pieces shared by the kernels that stream logits over the vocabulary (speculative verification, paper
// Sec. II-A; draft-side margin gate and candidates, Sec. III-B and III-C): vector loads of a logit row and the
// streaming softmax statistics.
#pragma once
#include "common.h"
#include "kernels.h"

namespace covspec {

template <int DT> struct LogitVec;
template <> struct LogitVec<DT_BF16> {
  static constexpr int N = 8;
  static __device__ __forceinline__ u32x4_t load_raw(const void* p, long i) { return *(const u32x4_t*)((const bf16_t*)p + i); }
  static __device__ __forceinline__ void unpack(const u32x4_t& w, float (&v)[8]) {
#pragma unroll
    for (int e = 0; e < 4; ++e) { v[2 * e] = bf16lo_to_f32(w[e]); v[2 * e + 1] = bf16hi_to_f32(w[e]); }
  }
  static __device__ __forceinline__ void load(const void* p, long i, float (&v)[8]) { unpack(load_raw(p, i), v); }
  static __device__ __forceinline__ double at(const void* p, long i) { return (double)bf16_to_f32(((const bf16_t*)p)[i]); }
};
template <> struct LogitVec<DT_F16> {
  static constexpr int N = 8;
  typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
  static __device__ __forceinline__ u32x4_t load_raw(const void* p, long i) { return *(const u32x4_t*)((const _Float16*)p + i); }
  static __device__ __forceinline__ void unpack(const u32x4_t& w, float (&v)[8]) {
    const half8_t h = __builtin_bit_cast(half8_t, w);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (float)h[e];
  }
  static __device__ __forceinline__ void load(const void* p, long i, float (&v)[8]) { unpack(load_raw(p, i), v); }
  static __device__ __forceinline__ double at(const void* p, long i) { return (double)(float)((const _Float16*)p)[i]; }
};
template <> struct LogitVec<DT_F32> {
  static constexpr int N = 4;
  static __device__ __forceinline__ u32x4_t load_raw(const void* p, long i) { return *(const u32x4_t*)((const float*)p + i); }
  static __device__ __forceinline__ void unpack(const u32x4_t& w, float (&v)[4]) {
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = __uint_as_float(w[e]);
  }
  static __device__ __forceinline__ void load(const void* p, long i, float (&v)[4]) { unpack(load_raw(p, i), v); }
  static __device__ __forceinline__ double at(const void* p, long i) { return (double)((const float*)p)[i]; }
};

// The streaming pass works in the base-2 domain: y = x * kLog2e (kLog2e the fp32 constant below, also used as
// the exact same number in the fp64 steps), terms 2^(y - c) against a reference c that is the largest y seen so
// far rounded to fp32.  One fused multiply-add forms y - c with a single rounding, so a term costs fma + exp2 +
// add.  The reference need not be the exact maximum: (c, sum) pairs combine exactly whatever c is.  kLog2e
// differs from log2(e) by 1.3e-8 relative, i.e. a temperature of 1 + 1.3e-8: below 1e-6 in any probability
// ratio for logits within +-50 of each other.
constexpr float kLog2e = 1.44269502f;

// running (reference, sum of 2^(y - reference)) of one thread, extended by a vector of N values
// returns the largest of the N values (NaN ignored)
template <int N>
__device__ __forceinline__ float online_add(float& c, float& s, const float (&v)[N]) {
  float vm = v[0];
#pragma unroll
  for (int e = 1; e < N; ++e) vm = fmaxf(vm, v[e]);
  const float cx = fmaxf(c, vm * kLog2e);
  const float cn = cx == -INFINITY ? 0.f : cx;   // only masked (-inf) words so far: any finite reference gives zeros
  float acc = s * __builtin_amdgcn_exp2f(c - cn);   // c = -inf at the start: 2^-inf = 0
#pragma unroll
  for (int e = 0; e < N; ++e) acc += __builtin_amdgcn_exp2f(__builtin_fmaf(v[e], kLog2e, -cn));
  c = cx;
  s = acc;
  return vm;
}

// combine of two (reference, sum) pairs of the base-2 domain
__device__ __forceinline__ void combine_pair(double& m, double& s, double m2, double s2) {
  const double mn = fmax(m, m2);
  s = (m == mn ? s : s * exp2(m - mn)) + (m2 == mn ? s2 : s2 * exp2(m2 - mn));
  m = mn;
}


// butterfly combine of (reference, sum) pairs over the wave; every lane ends with the wave's pair
__device__ __forceinline__ void wave_combine(double& m, double& s) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const double m2 = __shfl_xor(m, o, 64), s2 = __shfl_xor(s, o, 64);
    if (s2 > 0.0) {
      if (s > 0.0) combine_pair(m, s, m2, s2);
      else { m = m2; s = s2; }
    }
  }
}


// Workgroup combine of the threads' fp32 (reference, sum) pairs: each wave rescales to its largest reference
// (one fp32 exp2 per lane, relative error ~1e-7, inside the streaming sums' own), adds in fp64, and thread 0
// folds the waves the same way.  `red` holds 2 doubles per wave.  Contains a barrier: call uniformly; the
// result is valid in thread 0 only (sum 0 when every word was masked).
template <int WAVES>
__device__ __forceinline__ void block_combine(float c, float s, double (*red)[2], double& ref_out, double& sum_out) {
  const float cw = wave_max(c);
  const float f = cw == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(c - cw);
  const double sw = wave_sum((double)(s * f));
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  if (lane == 0) { red[wv][0] = (double)cw; red[wv][1] = sw; }
  __syncthreads();
  if (threadIdx.x == 0) {
    double cb = red[0][0];
#pragma unroll
    for (int k = 1; k < WAVES; ++k) cb = fmax(cb, red[k][0]);
    double tot = 0.0;
#pragma unroll
    for (int k = 0; k < WAVES; ++k)
      if (red[k][1] > 0.0) tot += red[k][1] * (double)__builtin_amdgcn_exp2f((float)(red[k][0] - cb));
    ref_out = cb;
    sum_out = tot;
  }
}

}  // namespace covspec
