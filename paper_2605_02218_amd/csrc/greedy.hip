// Greedy residual-update selection (a variant that is not in the paper; it replaces
// the rank-r SVD energy ranking of Sec. III-A.3 by k greedy picks).
//
// Pivoted Cholesky of the token Gram matrix G = Z Z^T in fp64: the residual squared
// norm of token i after projecting out the picked tokens is rho_i; each step picks
// argmax rho (decided on the fp32-rounded value, ties -> lower index), forms the new
// Cholesky column l = (G[:,p] - L L[p,:]^T) / sqrt(rho_p) and updates rho -= l^2.
// One 1024-thread workgroup per image; L is kept transposed (Lt[t][i]) so that the
// step-t dot products read it with unit stride across threads.
#include "common.h"
#include "kernels.h"

namespace covspec {

namespace {

constexpr int TPB = 1024;
constexpr int RPT = 4;  // rows per thread: n <= 4096

__global__ __launch_bounds__(TPB) void greedy_kernel(const double* __restrict__ G, int n, int nP, int k,
                                                      double* __restrict__ Lt, int32_t* __restrict__ order,
                                                      float* __restrict__ resid) {
  __shared__ double Lp[4096];
  __shared__ unsigned long long red[16];
  __shared__ double sh_piv;
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const double* Gb = G + (long)b * nP * nP;
  double* Ltb = Lt + (long)b * k * nP;

  double rho[RPT];
  bool picked[RPT];
#pragma unroll
  for (int s = 0; s < RPT; ++s) {
    const int i = tid + TPB * s;
    rho[s] = (i < n) ? Gb[(long)i * nP + i] : 0.0;
    picked[s] = !(i < n);
  }

  for (int t = 0; t < k; ++t) {
    // ---- argmax over the unpicked rows of float(rho), lowest index on ties
    unsigned long long best = 0ull;
#pragma unroll
    for (int s = 0; s < RPT; ++s) {
      if (!picked[s]) {
        const uint32_t i = (uint32_t)(tid + TPB * s);
        unsigned long long key = ((unsigned long long)float_order_key((float)rho[s]) << 32) | (0xFFFFFFFFu - i);
        best = key > best ? key : best;
      }
    }
    best = wave_max(best);
    if (lane == 0) red[w] = best;
    __syncthreads();
    best = red[0];
#pragma unroll
    for (int q = 1; q < TPB / 64; ++q) best = red[q] > best ? red[q] : best;
    const int p = (int)(0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull));
    if ((p & (TPB - 1)) == tid) {
#pragma unroll
      for (int s = 0; s < RPT; ++s)
        if (s == (p >> 10)) { sh_piv = rho[s]; picked[s] = true; }
    }
    for (int s = tid; s < t; s += TPB) Lp[s] = Ltb[(long)s * nP + p];
    __syncthreads();
    const double rp = sh_piv;
    const double piv = rp > 0.0 ? rp : 0.0;
    const double root = sqrt(piv);
    double dot[RPT];
#pragma unroll
    for (int s = 0; s < RPT; ++s) dot[s] = 0.0;
    for (int q = 0; q < t; ++q) {
      const double lp = Lp[q];
      const double* row = Ltb + (long)q * nP + tid;
#pragma unroll
      for (int s = 0; s < RPT; ++s)
        if (tid + TPB * s < n) dot[s] = fma(row[TPB * s], lp, dot[s]);
    }
#pragma unroll
    for (int s = 0; s < RPT; ++s) {
      const int i = tid + TPB * s;
      if (i < n) {
        const double col = piv > 0.0 ? (Gb[(long)p * nP + i] - dot[s]) / root : 0.0;
        Ltb[(long)t * nP + i] = col;
        rho[s] -= col * col;
      }
    }
    if (tid == 0) { order[(long)b * k + t] = p; resid[(long)b * k + t] = (float)rp; }
    __syncthreads();  // Lp, sh_piv and red are rewritten next step; Lt row t must be visible to all
  }
}

// idx_out[b,:] = ascending positions idx_m[b, picked]; pick_out[b,t] = idx_m[b, order[b,t]]
__global__ __launch_bounds__(TPB) void greedy_finish_kernel(const int32_t* __restrict__ order, const int32_t* __restrict__ idx_m,
                                                             int M, int k, int32_t* __restrict__ idx_out,
                                                             int32_t* __restrict__ pick_out) {
  __shared__ unsigned char flag[4096];
  __shared__ int wsum[17];
  const int b = blockIdx.x, tid = threadIdx.x;
  for (int i = tid; i < M; i += TPB) flag[i] = 0;
  __syncthreads();
  for (int t = tid; t < k; t += TPB) {
    const int p = order[(long)b * k + t];
    flag[p] = 1;
    if (pick_out) pick_out[(long)b * k + t] = idx_m[(long)b * M + p];
  }
  __syncthreads();
  const int per = (M + TPB - 1) / TPB, i0 = tid * per;
  int cnt = 0;
  for (int q = 0; q < per; ++q) { const int i = i0 + q; if (i < M && flag[i]) ++cnt; }
  int total;
  int pos = block_exscan_1024(cnt, wsum, &total);
  for (int q = 0; q < per; ++q) {
    const int i = i0 + q;
    if (i < M && flag[i]) idx_out[(long)b * k + pos++] = idx_m[(long)b * M + i];
  }
}

}  // namespace

hipError_t launch_greedy(const double* G, int B, int n, int nP, int k, double* Lt, int32_t* order, float* resid, hipStream_t st) {
  if (n > TPB * RPT || k > n || k > 4096) return hipErrorInvalidValue;
  hipLaunchKernelGGL(greedy_kernel, dim3(B), dim3(TPB), 0, st, G, n, nP, k, Lt, order, resid);
  return hipGetLastError();
}

hipError_t launch_greedy_finish(const int32_t* order, const int32_t* idx_m, int B, int M, int k, int32_t* idx_out,
                                int32_t* pick_out, hipStream_t st) {
  if (M > 4096) return hipErrorInvalidValue;
  hipLaunchKernelGGL(greedy_finish_kernel, dim3(B), dim3(TPB), 0, st, order, idx_m, M, k, idx_out, pick_out);
  return hipGetLastError();
}

}  // namespace covspec
