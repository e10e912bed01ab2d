// Block-wide exact top-m selection (pre-selection of the M best fused scores and
// the final "keep the B_vis largest energies", paper Sec. III-A.3).
//
// One 1024-thread workgroup per image, scores resident in LDS as order-preserving
// 32-bit keys.  A 4-pass, 8-bit radix select finds the m-th largest key exactly;
// elements above it are taken, elements equal to it are taken in index order until
// m is reached (ties -> lower index), and a block-wide scan compacts the winners in
// ascending index order.  All integer work: the result is a pure function of the
// fp32 score bits.
#include "common.h"
#include "kernels.h"

namespace covspec {

namespace {

constexpr int TPB = 1024;  // block_exscan_1024 assumes this
constexpr int MAXN = 16384;
constexpr int ITEMS = MAXN / TPB;

__global__ __launch_bounds__(TPB) void select_top_kernel(const float* __restrict__ scores, int n, int m,
                                                          const int32_t* __restrict__ map, int32_t* __restrict__ out) {
  __shared__ uint32_t keys[MAXN];
  __shared__ int hist[256];
  __shared__ int wsum[17];
  __shared__ uint32_t sh_prefix;
  __shared__ int sh_remaining;

  const int b = blockIdx.x;
  const float* s = scores + (long)b * n;
  for (int i = threadIdx.x; i < n; i += TPB) keys[i] = float_order_key(s[i]);
  if (threadIdx.x == 0) { sh_prefix = 0u; sh_remaining = m; }
  __syncthreads();

  uint32_t mask = 0u;
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (threadIdx.x < 256) hist[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t prefix = sh_prefix;
    for (int i = threadIdx.x; i < n; i += TPB) {
      uint32_t k = keys[i];
      if ((k & mask) == prefix) atomicAdd(&hist[(k >> shift) & 255u], 1);
    }
    __syncthreads();
    if (threadIdx.x < 64) {
      // lane l owns bins 255-4l .. 252-4l (descending); find the bin where the running count reaches `remaining`
      const int l = threadIdx.x;
      int c[4], tot = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) { c[q] = hist[255 - 4 * l - q]; tot += c[q]; }
      int inc = tot;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        int t = __shfl_up(inc, o, 64);
        if (l >= o) inc += t;
      }
      const int rem = sh_remaining;
      const int before = inc - tot;
      if (before < rem && rem <= inc) {
        int run = before;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if (run < rem && rem <= run + c[q]) {
            sh_prefix = prefix | ((uint32_t)(255 - 4 * l - q) << shift);
            sh_remaining = rem - run;
          }
          run += c[q];
        }
      }
    }
    mask |= 255u << shift;
    __syncthreads();
  }
  const uint32_t thr = sh_prefix;
  const int need_eq = sh_remaining;  // how many keys equal to thr are taken (lowest indices first)

  // blocked arrangement: thread t owns indices [t*per, (t+1)*per)
  const int per = (n + TPB - 1) / TPB;
  const int i0 = threadIdx.x * per;
  int eq_cnt = 0;
  for (int q = 0; q < per; ++q) { int i = i0 + q; if (i < n && keys[i] == thr) ++eq_cnt; }
  int total;
  int eq_before = block_exscan_1024(eq_cnt, wsum, &total);
  uint32_t take = 0u;  // bit q set => element i0+q selected (per <= 16)
  int cnt = 0;
  for (int q = 0; q < per; ++q) {
    int i = i0 + q;
    if (i >= n) break;
    uint32_t k = keys[i];
    bool sel = k > thr;
    if (k == thr) { sel = eq_before < need_eq; ++eq_before; }
    if (sel) { take |= 1u << q; ++cnt; }
  }
  int pos = block_exscan_1024(cnt, wsum, &total);
  for (int q = 0; q < per; ++q)
    if (take & (1u << q)) {
      int i = i0 + q;
      out[(long)b * m + pos] = map ? map[(long)b * n + i] : i;
      ++pos;
    }
}

}  // namespace

hipError_t launch_select_top(const float* scores, int B, int n, int m, const int32_t* map, int32_t* out, hipStream_t st) {
  if (n > MAXN || m > n || m < 1) return hipErrorInvalidValue;
  static_assert(ITEMS <= 32, "selection bitmask holds at most 32 items per thread");
  hipLaunchKernelGGL(select_top_kernel, dim3(B), dim3(TPB), 0, st, scores, n, m, map, out);
  return hipGetLastError();
}

}  // namespace covspec
