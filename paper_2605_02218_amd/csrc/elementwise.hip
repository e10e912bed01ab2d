// HBM-bound and small per-token kernels of the token-selection path:
// activity score, row norms, format conversion and splitting, the cosine-max
// and softmax epilogues, min-max fusion, gather.
#include <type_traits>

#include "common.h"
#include "kernels.h"

namespace covspec {

namespace {

// ---------------------------------------------------------------- 16-byte element loads
template <int DT> struct Vec;
template <> struct Vec<DT_BF16> {
  static constexpr int N = 8;
  __device__ static __forceinline__ void load(const void* base, long elem, float (&v)[8]) {
    u32x4_t r = *(const u32x4_t*)((const bf16_t*)base + elem);
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[2 * i] = bf16lo_to_f32(r[i]); v[2 * i + 1] = bf16hi_to_f32(r[i]); }
  }
  __device__ static __forceinline__ float load1(const void* base, long elem) { return bf16_to_f32(((const bf16_t*)base)[elem]); }
};
template <> struct Vec<DT_F32> {
  static constexpr int N = 4;
  __device__ static __forceinline__ void load(const void* base, long elem, float (&v)[4]) {
    f32x4_t r = *(const f32x4_t*)((const float*)base + elem);
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = r[i];
  }
  __device__ static __forceinline__ float load1(const void* base, long elem) { return ((const float*)base)[elem]; }
};

// ---------------------------------------------------------------- activity (paper Sec. III-A.2)
// One wave per token.  The wave walks the row in 16-byte-per-lane chunks and reads the K+1 slices of a
// chunk back to back, keeping the previous slice in registers, so every hidden element is read from
// HBM exactly once.  Squared differences accumulate in fp32 per (layer, lane) and are wave-reduced in a
// fixed order, so equal rows give bit-equal scores.  fp32 inputs accumulate in fp64, bf16 inputs in fp32
// (a difference of two bf16 values is exact in fp32).
template <int DT, int K, typename Acc>
__global__ __launch_bounds__(256) void activity_kernel(const void* __restrict__ hidden, float* __restrict__ s_act,
                                                        long tokens, int N, int d) {
  constexpr int V = Vec<DT>::N;
  const int lane = threadIdx.x & 63;
  const long token = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (token >= tokens) return;
  const long b = token / N, i = token - b * N;
  const long slice = (long)N * d;
  const long base = (b * (K + 1) * N + i) * (long)d;
  Acc acc[K];
#pragma unroll
  for (int l = 0; l < K; ++l) acc[l] = (Acc)0;
  for (int c = lane * V; c < d; c += 64 * V) {
    float prev[V], cur[V];
    Vec<DT>::load(hidden, base + c, prev);
#pragma unroll
    for (int l = 1; l <= K; ++l) {
      Vec<DT>::load(hidden, base + l * slice + c, cur);
#pragma unroll
      for (int e = 0; e < V; ++e) {
        const Acc df = (Acc)cur[e] - (Acc)prev[e];
        acc[l - 1] += df * df;
        prev[e] = cur[e];
      }
    }
  }
  double total = 0.0;
#pragma unroll
  for (int l = 0; l < K; ++l) total += sqrt((double)wave_sum(acc[l]));
  if (lane == 0) s_act[token] = (float)(total / K);
}

template <int DT>
hipError_t activity_dispatch(const void* hidden, float* s_act, long tokens, int N, int d, int K, hipStream_t st) {
  dim3 grid((unsigned)((tokens + 3) / 4)), block(256);
#define COVSPEC_ACT_CASE(KK) \
  case KK: hipLaunchKernelGGL((activity_kernel<DT, KK, typename std::conditional<DT == DT_F32, double, float>::type>), grid, block, 0, st, hidden, s_act, tokens, N, d); break;
  switch (K) {
    COVSPEC_ACT_CASE(1) COVSPEC_ACT_CASE(2) COVSPEC_ACT_CASE(3) COVSPEC_ACT_CASE(4)
    COVSPEC_ACT_CASE(5) COVSPEC_ACT_CASE(6) COVSPEC_ACT_CASE(7) COVSPEC_ACT_CASE(8)
    default: return hipErrorInvalidValue;
  }
#undef COVSPEC_ACT_CASE
  return hipGetLastError();
}

// ---------------------------------------------------------------- row norms
template <typename In> __device__ __forceinline__ double load_as_f64(const In* p, long i);
template <> __device__ __forceinline__ double load_as_f64<bf16_t>(const bf16_t* p, long i) { return (double)bf16_to_f32(p[i]); }
template <> __device__ __forceinline__ double load_as_f64<float>(const float* p, long i) { return (double)p[i]; }
template <> __device__ __forceinline__ double load_as_f64<double>(const double* p, long i) { return p[i]; }

// one wave per row; Out = float accumulates in fp32, Out = double in fp64
template <typename In, typename Out>
__global__ __launch_bounds__(256) void row_norm2_kernel(const In* __restrict__ x, Out* __restrict__ out, long rows, int d) {
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  Out acc = (Out)0;
  for (int c = lane; c < d; c += 64) {
    const Out v = (Out)load_as_f64<In>(x, row * d + c);
    acc += v * v;
  }
  acc = wave_sum(acc);
  if (lane == 0) out[row] = acc;
}

// ---------------------------------------------------------------- transpose
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T* __restrict__ in, T* __restrict__ out, int rows, int cols) {
  __shared__ T tile[64][65];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  for (int r = ty; r < 64; r += 4)
    if (r0 + r < rows && c0 + tx < cols) tile[r][tx] = in[(long)(r0 + r) * cols + c0 + tx];
  __syncthreads();
  for (int c = ty; c < 64; c += 4)
    if (c0 + c < cols && r0 + tx < rows) out[(long)(c0 + c) * rows + r0 + tx] = tile[tx][c];
}

// ---------------------------------------------------------------- conversion / splitting
template <typename In, typename Out>
__global__ void convert_kernel(const In* __restrict__ src, Out* __restrict__ dst, long n) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = (Out)load_as_f64<In>(src, i);
}

__device__ __forceinline__ float sum_planes(const float* src, int planes, long plane_stride, long i) {
  float v = src[i];
  for (int p = 1; p < planes; ++p) v += src[p * plane_stride + i];
  return v;
}

// V elements of a row per thread (V = 4 when d % 4 == 0 and the planes and the output start on 16- / 8-byte boundaries:
// one 16-byte load per plane and one 8-byte store per output plane; else V = 1).  The sum over the planes is taken in
// plane order per element, the same in both widths.
template <int V>
__global__ __launch_bounds__(256) void sum_split3_kernel(const float* __restrict__ src, int planes, long plane_stride, long rows, int d,
                                                         long rpg, bf16_t* __restrict__ out) {
  const long i = ((long)blockIdx.x * blockDim.x + threadIdx.x) * V;
  if (i >= rows * d) return;
  const long r = i / d;
  const int c = (int)(i - r * d);
  float v[V];
  if (V == 4) {
    const f32x4_t x = *(const f32x4_t*)(src + i);
#pragma unroll
    for (int e = 0; e < V; ++e) v[e] = x[e];
    for (int p = 1; p < planes; ++p) {
      const f32x4_t y = *(const f32x4_t*)(src + p * plane_stride + i);
#pragma unroll
      for (int e = 0; e < V; ++e) v[e] += y[e];
    }
  } else {
    v[0] = sum_planes(src, planes, plane_stride, i);
  }
  bf16_t hi[V], mid[V], lo[V];
#pragma unroll
  for (int e = 0; e < V; ++e) {
    hi[e] = f32_to_bf16_rne(v[e]);
    const float r1 = v[e] - bf16_to_f32(hi[e]);  // exact
    mid[e] = f32_to_bf16_rne(r1);
    const float r2 = r1 - bf16_to_f32(mid[e]);   // exact
    lo[e] = f32_to_bf16_rne(r2);
  }
  const long g = r / rpg, j = r - g * rpg;
  bf16_t* o0 = out + ((g * 3 + 0) * rpg + j) * d + c;
  bf16_t* o1 = out + ((g * 3 + 1) * rpg + j) * d + c;
  bf16_t* o2 = out + ((g * 3 + 2) * rpg + j) * d + c;
  if (V == 4) {
    typedef unsigned short u16x4_t __attribute__((ext_vector_type(4)));
    *(u16x4_t*)o0 = (u16x4_t){hi[0], hi[1], hi[2], hi[3]};
    *(u16x4_t*)o1 = (u16x4_t){mid[0], mid[1], mid[2], mid[3]};
    *(u16x4_t*)o2 = (u16x4_t){lo[0], lo[1], lo[2], lo[3]};
  } else {
    *o0 = hi[0];
    *o1 = mid[0];
    *o2 = lo[0];
  }
}

// ---------------------------------------------------------------- cosine-max epilogue (paper Sec. III-A.1)
// s_query[token] = max_j dot_j / max(|e(v)| |e(q_j)|, 1e-30), dot_j = the sum of the logit planes of keyword j.  The
// scalar arithmetic is fp64 so that the only error left in the score is that of the fp32-accumulated contractions
// feeding it.  Four lanes per token, 64 tokens of one image per workgroup: the keywords' 1 / |e(q_j)| are formed once
// per workgroup (LDS) and a token's |e(v)| once, so that a keyword costs a token one multiplication
// (max_j dot_j / (|v| |q_j|) = (max_j dot_j / |q_j|) / |v|; a wave per token with a square root and a division per
// keyword was bound by those: 156 us for workload 5 where its 283 MB of logits are 50 us of HBM time).  Where the
// floor could bind (|v| |q_j| < 1e-30 for some keyword that is not a zero vector) the token takes the literal formula.
template <typename F>
__global__ __launch_bounds__(256) void cosine_max_kernel(const F* __restrict__ logits, int planes,
                                                          const F* __restrict__ vnorm2, int nparts,
                                                          const F* __restrict__ qnorm2, float* __restrict__ s_query,
                                                          int N, int T) {
  extern __shared__ double cm_lds[];    // [T] 1 / |e(q_j)| (0 for a zero vector), then the smallest non-zero |e(q_j)|
  double* rq = cm_lds;
  double* minq = cm_lds + T;
  const int tid = threadIdx.x, q = tid & 3;
  const int b = blockIdx.y;
  if (tid == 0) *minq = 1e300;
  __syncthreads();
  double mine = 1e300;
  for (int j = tid; j < T; j += 256) {
    const double sq = sqrt((double)qnorm2[(long)b * T + j]);
    rq[j] = sq > 0.0 ? 1.0 / sq : 0.0;
    if (sq > 0.0) mine = fmin(mine, sq);
  }
  mine = wave_min(mine);
  if ((tid & 63) == 0 && mine < 1e300) atomicMin((unsigned long long*)minq, (unsigned long long)__double_as_longlong(mine));   // positive doubles order like their bits
  __syncthreads();
  const double smallest = *minq;
  const int n = blockIdx.x * 64 + (tid >> 2);
  if (n >= N) return;      // whole quads leave together
  const long token = (long)b * N + n;
  double n2 = 0.0;
  for (int t = q; t < nparts; t += 4) n2 += (double)vnorm2[token * nparts + t];
  n2 += __shfl_xor(n2, 1, 64);
  n2 += __shfl_xor(n2, 2, 64);
  const double nv = sqrt(n2);
  const F* L = logits + token * (long)planes * T;
  double best = -INFINITY;
  if (nv * smallest >= 1e-30) {
    if (std::is_same<F, float>::value && (T & 3) == 0 && (((uintptr_t)logits) & 15) == 0) {
      for (int j0 = 4 * q; j0 < T; j0 += 16) {
        f32x4_t x = *(const f32x4_t*)((const float*)L + j0);
        double d0 = x[0], d1 = x[1], d2 = x[2], d3 = x[3];
        for (int s_ = 1; s_ < planes; ++s_) {
          x = *(const f32x4_t*)((const float*)L + (long)s_ * T + j0);
          d0 += x[0]; d1 += x[1]; d2 += x[2]; d3 += x[3];
        }
        best = fmax(best, fmax(fmax(d0 * rq[j0], d1 * rq[j0 + 1]), fmax(d2 * rq[j0 + 2], d3 * rq[j0 + 3])));
      }
    } else {
      for (int j = q; j < T; j += 4) {
        double dot = (double)L[j];
        for (int s_ = 1; s_ < planes; ++s_) dot += (double)L[(long)s_ * T + j];
        best = fmax(best, dot * rq[j]);
      }
    }
    best = best / nv;     // nv > 0 here
  } else {
    for (int j = q; j < T; j += 4) {
      double dot = (double)L[j];
      for (int s_ = 1; s_ < planes; ++s_) dot += (double)L[(long)s_ * T + j];
      const double den = nv * sqrt((double)qnorm2[(long)b * T + j]);
      best = fmax(best, dot / fmax(den, 1e-30));
    }
  }
  best = fmax(best, __shfl_xor(best, 1, 64));
  best = fmax(best, __shfl_xor(best, 2, 64));
  if (q == 0) s_query[token] = (float)best;
}

// ---------------------------------------------------------------- softmax relevance (variant)
// stats[row] = (max_i scale*S[row,i], 1 / sum_i exp(scale*S[row,i] - max)); one wave per row, one pass: every
// lane keeps a running (maximum, sum) of its elements and rescales the sum when the maximum moves.
template <typename F>
__global__ __launch_bounds__(256) void softmax_stats_kernel(const F* __restrict__ S, double2* __restrict__ stats,
                                                             long rows, int N, double scale) {
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const F* p = S + row * (long)N;
  F m = -INFINITY;
  double z = 0.0;
  for (int i = lane; i < N; i += 64) {
    const F v = p[i] * (F)scale;
    if (v > m) { z *= (double)exp(m - v); m = v; }      // m = -inf at first: exp(-inf) = 0
    z += (double)exp(v - m);
  }
  const F mw = wave_max(m);
  z *= (m == -INFINITY) ? 0.0 : (double)exp(m - mw);
  z = wave_sum(z);
  if (lane == 0) stats[row] = make_double2((double)mw, 1.0 / z);
}

// s_query[b,i] = (1/HT) sum_{row < HT} exp(scale*S[b,row,i] - max_row) / Z_row, rows added in order (four
// interleaved partial sums, so that four loads are in flight).
template <typename F>
__global__ __launch_bounds__(256) void softmax_mean_kernel(const F* __restrict__ S, const double2* __restrict__ stats,
                                                            float* __restrict__ s_query, int HT, int N, double scale) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  const int b = blockIdx.y;
  if (i >= N) return;
  const F* p = S + (long)b * HT * N + i;
  const double2* st = stats + (long)b * HT;
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
  int r = 0;
  for (; r + 4 <= HT; r += 4) {
    F v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = p[(long)(r + u) * N];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const double2 mz = st[r + u];
      acc[u] = fma((double)exp(v[u] * (F)scale - (F)mz.x), mz.y, acc[u]);
    }
  }
  for (; r < HT; ++r) {
    const double2 mz = st[r];
    acc[0] = fma((double)exp(p[(long)r * N] * (F)scale - (F)mz.x), mz.y, acc[0]);
  }
  s_query[(long)b * N + i] = (float)(((acc[0] + acc[1]) + (acc[2] + acc[3])) / HT);
}

// fp32 logits with N a multiple of 4 (the bf16 workloads): the same two passes with 16-byte loads, base-2
// exponentials (one v_exp_f32 each) and fp32 partial sums; fp64 only where partial results are combined.
// stats[row] = (max_i log2(e)*scale*S[row,i], 1 / sum_i 2^(log2(e)*scale*S[row,i] - max)).
constexpr float kLog2eF = 1.44269504f;

__global__ __launch_bounds__(256) void softmax_stats4_kernel(const float4* __restrict__ S, double2* __restrict__ stats, long rows,
                                                              int N4, float sl2) {
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const float4* p = S + row * (long)N4;
  float m = -INFINITY, z = 0.f;
  for (int c = lane; c < N4; c += 64) {
    const float4 x = p[c];
    const float a = x.x * sl2, b = x.y * sl2, cc = x.z * sl2, d = x.w * sl2;
    const float mx = fmaxf(fmaxf(a, b), fmaxf(cc, d));
    if (mx > m) { z *= __builtin_amdgcn_exp2f(m - mx); m = mx; }     // m = -inf at first: 2^-inf = 0
    z += (__builtin_amdgcn_exp2f(a - m) + __builtin_amdgcn_exp2f(b - m)) + (__builtin_amdgcn_exp2f(cc - m) + __builtin_amdgcn_exp2f(d - m));
  }
  const float mw = wave_max(m);
  double zd = (m == -INFINITY) ? 0.0 : (double)z * (double)__builtin_amdgcn_exp2f(m - mw);
  zd = wave_sum(zd);
  if (lane == 0) stats[row] = make_double2((double)mw, 1.0 / zd);
}

// part[seg][b][i] = sum over the rows of segment seg of 2^(sl2*S[b,row,i] - max_row) / Z_row; a thread owns four
// neighbouring tokens and keeps four rows (64 bytes) in flight.
__global__ __launch_bounds__(256) void softmax_mean4_part_kernel(const float4* __restrict__ S, const double2* __restrict__ stats,
                                                                  double* __restrict__ part, int HT, int N4, int seg_rows, float sl2) {
  const int i4 = blockIdx.x * blockDim.x + threadIdx.x;
  const int b = blockIdx.y, seg = blockIdx.z, B = gridDim.y;
  if (i4 >= N4) return;
  const int r0 = seg * seg_rows, r1 = min(HT, r0 + seg_rows);
  const float4* p = S + (long)b * HT * N4 + i4;
  const double2* st = stats + (long)b * HT;
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  int r = r0;
  for (; r + 4 <= r1; r += 4) {
    float4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = p[(long)(r + u) * N4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const double2 mz = st[r + u];
      const float mref = (float)mz.x, rz = (float)mz.y;
      a0 = fmaf(__builtin_amdgcn_exp2f(fmaf(v[u].x, sl2, -mref)), rz, a0);
      a1 = fmaf(__builtin_amdgcn_exp2f(fmaf(v[u].y, sl2, -mref)), rz, a1);
      a2 = fmaf(__builtin_amdgcn_exp2f(fmaf(v[u].z, sl2, -mref)), rz, a2);
      a3 = fmaf(__builtin_amdgcn_exp2f(fmaf(v[u].w, sl2, -mref)), rz, a3);
    }
  }
  for (; r < r1; ++r) {
    const float4 v = p[(long)r * N4];
    const double2 mz = st[r];
    const float mref = (float)mz.x, rz = (float)mz.y;
    a0 = fmaf(__builtin_amdgcn_exp2f(fmaf(v.x, sl2, -mref)), rz, a0);
    a1 = fmaf(__builtin_amdgcn_exp2f(fmaf(v.y, sl2, -mref)), rz, a1);
    a2 = fmaf(__builtin_amdgcn_exp2f(fmaf(v.z, sl2, -mref)), rz, a2);
    a3 = fmaf(__builtin_amdgcn_exp2f(fmaf(v.w, sl2, -mref)), rz, a3);
  }
  double* out = part + (((long)seg * B + b) * N4 + i4) * 4;
  out[0] = a0; out[1] = a1; out[2] = a2; out[3] = a3;
}

// s_query[b,i] = (sum over the segments, in order, of part[seg][b][i]) / HT
__global__ __launch_bounds__(256) void softmax_mean_finish_kernel(const double* __restrict__ part, float* __restrict__ s_query, long BN,
                                                                   int segs, int HT) {
  const long e = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= BN) return;
  double s = 0.0;
  for (int g = 0; g < segs; ++g) s += part[(long)g * BN + e];
  s_query[e] = (float)(s / HT);
}

// ---------------------------------------------------------------- min-max + fuse (paper fusion equation)
__device__ __forceinline__ void block_minmax(float& lo, float& hi, float* red) {
  lo = wave_min(lo);
  hi = wave_max(hi);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) { red[w] = lo; red[32 + w] = hi; }
  __syncthreads();
  lo = red[0]; hi = red[32];
  for (int k = 1; k < nw; ++k) { lo = fminf(lo, red[k]); hi = fmaxf(hi, red[32 + k]); }
}

__global__ __launch_bounds__(1024) void fuse_kernel(const float* __restrict__ s_query, const float* __restrict__ s_act,
                                                     float* __restrict__ s_fused, int N, float lambda) {
  __shared__ float red[64];
  const long off = (long)blockIdx.x * N;
  float qlo = INFINITY, qhi = -INFINITY, alo = INFINITY, ahi = -INFINITY;
  for (int i = threadIdx.x; i < N; i += blockDim.x) {
    float q = s_query[off + i];
    qlo = fminf(qlo, q); qhi = fmaxf(qhi, q);
    if (s_act) { float a = s_act[off + i]; alo = fminf(alo, a); ahi = fmaxf(ahi, a); }
  }
  block_minmax(qlo, qhi, red);
  if (s_act) block_minmax(alo, ahi, red);
  const double lam = (double)lambda;
  for (int i = threadIdx.x; i < N; i += blockDim.x) {
    double q = (qhi == qlo) ? 0.0 : ((double)s_query[off + i] - (double)qlo) / ((double)qhi - (double)qlo);
    double f = q;
    if (s_act) {
      double a = (ahi == alo) ? 0.0 : ((double)s_act[off + i] - (double)alo) / ((double)ahi - (double)alo);
      f = lam * q + (1.0 - lam) * a;
    }
    s_fused[off + i] = (float)f;
  }
}

// ---------------------------------------------------------------- gather
__global__ __launch_bounds__(256) void gather_rows_kernel(const unsigned char* __restrict__ X, const int32_t* __restrict__ idx,
                                                           unsigned char* __restrict__ out, int N, int k, long row_bytes) {
  const long row = blockIdx.x;  // b*k + j
  const long b = row / k;
  const long src = (b * N + idx[row]) * row_bytes;
  const long dst = row * row_bytes;
  for (long o = (long)threadIdx.x * 16; o < row_bytes; o += 256 * 16)
    *(u32x4_t*)(out + dst + o) = *(const u32x4_t*)(X + src + o);
}

__global__ void fill_zero_kernel(u32x4_t* p, long n16) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const u32x4_t z = {0u, 0u, 0u, 0u};
  for (; i < n16; i += (long)gridDim.x * blockDim.x) p[i] = z;
}

inline unsigned blocks_for(long n, int per) { return (unsigned)((n + per - 1) / per); }

__global__ __launch_bounds__(256) void random_scores_kernel(float* __restrict__ out, int B, int N, uint32_t seed, int image0) {
  const long e = (long)blockIdx.x * 256 + threadIdx.x;
  if (e >= (long)B * N) return;
  const unsigned long long b = (unsigned long long)(e / N), i = (unsigned long long)(e - (long)b * N);
  // image0: index of this call's first image in the caller's batch (a ragged batch is worked off in runs)
  unsigned long long z = (unsigned long long)seed * 0x9E3779B97F4A7C15ull + (((b + (unsigned long long)image0) << 32) | i) + 0x632BE59BD9B4E019ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z ^= z >> 31;
  out[e] = (float)(unsigned int)(z >> 40) * 0x1p-24f;
}

__global__ void fill_int_kernel(int* __restrict__ p, int n, int value) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = value;
}

}  // namespace

hipError_t launch_transpose(const void* in, void* out, int rows, int cols, int dtype, hipStream_t st) {
  dim3 grid((cols + 63) / 64, (rows + 63) / 64), block(256);
  if (dtype == DT_BF16) hipLaunchKernelGGL((transpose_kernel<bf16_t>), grid, block, 0, st, (const bf16_t*)in, (bf16_t*)out, rows, cols);
  else hipLaunchKernelGGL((transpose_kernel<float>), grid, block, 0, st, (const float*)in, (float*)out, rows, cols);
  return hipGetLastError();
}

hipError_t launch_activity(const void* hidden, float* s_act, int B, int N, int d, int K, int dtype, hipStream_t st) {
  long tokens = (long)B * N;
  return dtype == DT_BF16 ? activity_dispatch<DT_BF16>(hidden, s_act, tokens, N, d, K, st)
                          : activity_dispatch<DT_F32>(hidden, s_act, tokens, N, d, K, st);
}

hipError_t launch_row_norm2(const void* x, int in_type, void* out, bool out_f64, long rows, int d, hipStream_t st) {
  dim3 grid(blocks_for(rows, 4)), block(256);
  if (in_type == IN_BF16 && !out_f64) hipLaunchKernelGGL((row_norm2_kernel<bf16_t, float>), grid, block, 0, st, (const bf16_t*)x, (float*)out, rows, d);
  else if (in_type == IN_F32 && !out_f64) hipLaunchKernelGGL((row_norm2_kernel<float, float>), grid, block, 0, st, (const float*)x, (float*)out, rows, d);
  else if (in_type == IN_F32 && out_f64) hipLaunchKernelGGL((row_norm2_kernel<float, double>), grid, block, 0, st, (const float*)x, (double*)out, rows, d);
  else if (in_type == IN_F64 && out_f64) hipLaunchKernelGGL((row_norm2_kernel<double, double>), grid, block, 0, st, (const double*)x, (double*)out, rows, d);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_convert(const void* src, int in_type, void* dst, bool out_f64, long n, hipStream_t st) {
  dim3 grid(blocks_for(n, 256)), block(256);
  if (in_type == IN_BF16 && !out_f64) hipLaunchKernelGGL((convert_kernel<bf16_t, float>), grid, block, 0, st, (const bf16_t*)src, (float*)dst, n);
  else if (in_type == IN_F32 && out_f64) hipLaunchKernelGGL((convert_kernel<float, double>), grid, block, 0, st, (const float*)src, (double*)dst, n);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_sum_split3(const float* src, int planes, long plane_stride, long rows, int d, long rows_per_group,
                             unsigned short* out, hipStream_t st) {
  const bool wide = d % 4 == 0 && plane_stride % 4 == 0 && ((uintptr_t)src & 15) == 0 && ((uintptr_t)out & 7) == 0;
  dim3 block(256);
  if (wide) hipLaunchKernelGGL(sum_split3_kernel<4>, dim3(blocks_for(rows * d / 4, 256)), block, 0, st, src, planes, plane_stride, rows, d, rows_per_group, out);
  else hipLaunchKernelGGL(sum_split3_kernel<1>, dim3(blocks_for(rows * d, 256)), block, 0, st, src, planes, plane_stride, rows, d, rows_per_group, out);
  return hipGetLastError();
}

hipError_t launch_cosine_max(const void* logits, int planes, const void* vnorm2, int nparts, const void* qnorm2, bool f64,
                             float* s_query, int B, int N, int T, hipStream_t st) {
  if (B <= 0 || N <= 0) return hipSuccess;
  dim3 grid((unsigned)((N + 63) / 64), (unsigned)B), block(256);
  const size_t lds = (size_t)(T + 1) * sizeof(double);
  if (lds > 48 * 1024) return hipErrorInvalidValue;     // more than 6143 query keywords
  if (f64) hipLaunchKernelGGL((cosine_max_kernel<double>), grid, block, lds, st, (const double*)logits, planes, (const double*)vnorm2, nparts, (const double*)qnorm2, s_query, N, T);
  else hipLaunchKernelGGL((cosine_max_kernel<float>), grid, block, lds, st, (const float*)logits, planes, (const float*)vnorm2, nparts, (const float*)qnorm2, s_query, N, T);
  return hipGetLastError();
}

// The fast path needs fp32 logits, N % 4 == 0 and `part` scratch of softmax_scratch_bytes(B, N) bytes.
size_t softmax_scratch_bytes(int B, int N) { return (size_t)32 * B * N * sizeof(double); }

hipError_t launch_softmax_stats(const void* S, bool f64, void* stats, long rows, int N, double scale, bool base2, hipStream_t st) {
  dim3 grid(blocks_for(rows, 4)), block(256);
  if (f64) hipLaunchKernelGGL((softmax_stats_kernel<double>), grid, block, 0, st, (const double*)S, (double2*)stats, rows, N, scale);
  else if (base2) hipLaunchKernelGGL(softmax_stats4_kernel, grid, block, 0, st, (const float4*)S, (double2*)stats, rows, N / 4, (float)scale * kLog2eF);
  else hipLaunchKernelGGL((softmax_stats_kernel<float>), grid, block, 0, st, (const float*)S, (double2*)stats, rows, N, scale);
  return hipGetLastError();
}

bool softmax_base2(bool f64, int N) { return !f64 && N % 4 == 0; }

hipError_t launch_softmax_mean(const void* S, bool f64, const void* stats, float* s_query, int B, int HT, int N, double scale,
                               void* part, hipStream_t st) {
  if (softmax_base2(f64, N) && part) {
    const int N4 = N / 4, gx = (N4 + 255) / 256;
    // row segments: enough workgroups for eight waves per SIMD, at most 32 segments of at least 32 rows
    int segs = (2048 + gx * B - 1) / (gx * B);
    const int most = HT / 32 > 0 ? HT / 32 : 1;
    segs = segs > 32 ? 32 : segs;
    segs = segs > most ? most : segs;
    const int seg_rows = (HT + segs - 1) / segs;
    segs = (HT + seg_rows - 1) / seg_rows;
    hipLaunchKernelGGL(softmax_mean4_part_kernel, dim3(gx, B, segs), dim3(256), 0, st, (const float4*)S, (const double2*)stats,
                       (double*)part, HT, N4, seg_rows, (float)scale * kLog2eF);
    const long BN = (long)B * N;
    hipLaunchKernelGGL(softmax_mean_finish_kernel, dim3(blocks_for(BN, 256)), dim3(256), 0, st, (const double*)part, s_query, BN, segs, HT);
    return hipGetLastError();
  }
  dim3 grid((N + 255) / 256, B), block(256);
  if (f64) hipLaunchKernelGGL((softmax_mean_kernel<double>), grid, block, 0, st, (const double*)S, (const double2*)stats, s_query, HT, N, scale);
  else hipLaunchKernelGGL((softmax_mean_kernel<float>), grid, block, 0, st, (const float*)S, (const double2*)stats, s_query, HT, N, scale);
  return hipGetLastError();
}

hipError_t launch_fuse(const float* s_query, const float* s_act, float* s_fused, int B, int N, float lambda, hipStream_t st) {
  hipLaunchKernelGGL(fuse_kernel, dim3(B), dim3(1024), 0, st, s_query, s_act, s_fused, N, lambda);
  return hipGetLastError();
}

hipError_t launch_gather_rows(const void* X, const int32_t* idx, void* out, int B, int N, int k, long row_bytes, hipStream_t st) {
  hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)((long)B * k)), dim3(256), 0, st, (const unsigned char*)X, idx,
                     (unsigned char*)out, N, k, row_bytes);
  return hipGetLastError();
}

hipError_t launch_random_scores(float* out, int B, int N, uint32_t seed, int image0, hipStream_t stream) {
  const long total = (long)B * N;
  if (total <= 0) return hipSuccess;
  hipLaunchKernelGGL(random_scores_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, out, B, N, seed, image0);
  return hipGetLastError();
}

hipError_t launch_fill_int(int* p, int n, int value, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill_int_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p, n, value);
  return hipGetLastError();
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st) {
  long n16 = (long)(bytes / 16);
  if (n16 == 0) return hipSuccess;
  unsigned blocks = (unsigned)((n16 + 255) / 256);
  if (blocks > 65536u) blocks = 65536u;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, st, (u32x4_t*)p, n16);
  return hipGetLastError();
}

}  // namespace covspec
