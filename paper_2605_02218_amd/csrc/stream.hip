// Data movement of the streaming (frame by frame) selection: the candidates of a frame are the tokens kept so far
// followed by the frame's pre-selected tokens, the kept tokens' Gram matrix is carried from frame to frame, and after
// the decision rows, ids and the Gram block of the survivors are compacted into the next state.  (The frame-by-frame
// form is not in the paper; each frame is one low-rank step of its Sec. III-A.3 on the candidate set.)
#include "common.h"
#include "kernels.h"

namespace covspec {

namespace {

// idc[b, i] = i < n_keep ? id_in[b, i] : id_base + idx_f[b, i - n_keep]      (n_c = n_keep + m candidates)
__global__ __launch_bounds__(256) void stream_ids_kernel(const int32_t* __restrict__ id_in, const int32_t* __restrict__ idx_f,
                                                          int32_t* __restrict__ idc, int n_keep, int m, int kcap, int id_base) {
  const int b = blockIdx.y, i = blockIdx.x * 256 + threadIdx.x, n_c = n_keep + m;
  if (i >= n_c) return;
  idc[(long)b * n_c + i] = i < n_keep ? id_in[(long)b * kcap + i] : id_base + idx_f[(long)b * m + (i - n_keep)];
}

// dst[b][i][j] = src[b][i][j] for i, j < n
__global__ __launch_bounds__(256) void copy_block_kernel(double* __restrict__ dst, long dpitch, long dstride,
                                                          const double* __restrict__ src, long spitch, long sstride, int n) {
  const int b = blockIdx.z, i = blockIdx.y, j = blockIdx.x * 256 + threadIdx.x;
  if (j < n) dst[(long)b * dstride + (long)i * dpitch + j] = src[(long)b * sstride + (long)i * spitch + j];
}

// G[b][j][i] = G[b][i][j] for n0 <= i < n1, j < n0   (the new rows' block against the kept tokens, transposed)
__global__ __launch_bounds__(256) void mirror_block_kernel(double* G, long pitch, long stride, int n0, int n1) {
  __shared__ double tile[32][33];
  double* Gb = G + (long)blockIdx.z * stride;
  const int i0 = n0 + blockIdx.y * 32, j0 = blockIdx.x * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;      // 32 x 8
  for (int r = ty; r < 32; r += 8) {
    const int i = i0 + r, j = j0 + tx;
    tile[r][tx] = (i < n1 && j < n0) ? Gb[(long)i * pitch + j] : 0.0;
  }
  __syncthreads();
  for (int r = ty; r < 32; r += 8) {
    const int j = j0 + r, i = i0 + tx;
    if (i < n1 && j < n0) Gb[(long)j * pitch + i] = tile[tx][r];
  }
}

// Row j of the next state of image b = candidate sel[b, j] (sel == nullptr: candidate j): a kept row of Z_in or row
// idx_f[...] of the frame, copied in 16-byte pieces; its id travels with it.
__global__ __launch_bounds__(256) void stream_compact_rows_kernel(const uint4* __restrict__ Z_in, const uint4* __restrict__ X,
                                                                   const int32_t* __restrict__ idx_f, const int32_t* __restrict__ sel,
                                                                   const int32_t* __restrict__ idc, uint4* __restrict__ Z_out,
                                                                   int32_t* __restrict__ id_out, int n_keep, int m, int kcap, int N,
                                                                   int n_out, long row16) {
  const int b = blockIdx.y, j = blockIdx.x, n_c = n_keep + m;
  const int cand = sel ? sel[(long)b * n_out + j] : j;
  if ((unsigned)cand >= (unsigned)n_c) return;                 // cannot happen with a consistent selection; never index with it
  const uint4* src;
  if (cand < n_keep) src = Z_in + ((long)b * kcap + cand) * row16;
  else {
    const int pos = idx_f[(long)b * m + (cand - n_keep)];
    if ((unsigned)pos >= (unsigned)N) return;
    src = X + ((long)b * N + pos) * row16;
  }
  uint4* dst = Z_out + ((long)b * kcap + j) * row16;
  for (long e = threadIdx.x; e < row16; e += 256) dst[e] = src[e];
  if (threadIdx.x == 0) id_out[(long)b * kcap + j] = idc[(long)b * n_c + cand];
}

// G_out[b][i][j] = Gc[b][sel_i][sel_j]   (sel == nullptr: the leading n_out x n_out block)
__global__ __launch_bounds__(256) void gather_sym_kernel(const double* __restrict__ Gc, long pitch, long stride,
                                                          const int32_t* __restrict__ sel, double* __restrict__ G_out, int kcap,
                                                          int n_out, int n_c) {
  const int b = blockIdx.z, i = blockIdx.y, j = blockIdx.x * 256 + threadIdx.x;
  if (j >= n_out) return;
  const int si = sel ? sel[(long)b * n_out + i] : i, sj = sel ? sel[(long)b * n_out + j] : j;
  if ((unsigned)si >= (unsigned)n_c || (unsigned)sj >= (unsigned)n_c) return;
  G_out[((long)b * kcap + i) * kcap + j] = Gc[(long)b * stride + (long)si * pitch + sj];
}

}  // namespace

hipError_t launch_stream_ids(const int32_t* id_in, const int32_t* idx_f, int32_t* idc, int B, int n_keep, int m, int kcap,
                             int id_base, hipStream_t st) {
  hipLaunchKernelGGL(stream_ids_kernel, dim3((n_keep + m + 255) / 256, B), dim3(256), 0, st, id_in, idx_f, idc, n_keep, m, kcap, id_base);
  return hipGetLastError();
}

hipError_t launch_copy_block(double* dst, long dpitch, long dstride, const double* src, long spitch, long sstride, int n, int B,
                             hipStream_t st) {
  if (n < 1) return hipSuccess;
  hipLaunchKernelGGL(copy_block_kernel, dim3((n + 255) / 256, n, B), dim3(256), 0, st, dst, dpitch, dstride, src, spitch, sstride, n);
  return hipGetLastError();
}

hipError_t launch_mirror_block(double* G, long pitch, long stride, int n0, int n1, int B, hipStream_t st) {
  if (n0 < 1 || n1 <= n0) return hipSuccess;
  hipLaunchKernelGGL(mirror_block_kernel, dim3((n0 + 31) / 32, (n1 - n0 + 31) / 32, B), dim3(256), 0, st, G, pitch, stride, n0, n1);
  return hipGetLastError();
}

hipError_t launch_stream_compact(const void* Z_in, const void* X, const int32_t* idx_f, const int32_t* sel, const int32_t* idc,
                                 const double* Gc, long pitch, long stride, void* Z_out, int32_t* id_out, double* G_out, int B,
                                 int n_keep, int m, int kcap, int N, int n_out, long row_bytes, hipStream_t st) {
  if (row_bytes % 16 != 0 || n_out < 1 || n_out > kcap) return hipErrorInvalidValue;
  hipLaunchKernelGGL(stream_compact_rows_kernel, dim3(n_out, B), dim3(256), 0, st, (const uint4*)Z_in, (const uint4*)X, idx_f, sel, idc,
                     (uint4*)Z_out, id_out, n_keep, m, kcap, N, n_out, row_bytes / 16);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(gather_sym_kernel, dim3((n_out + 255) / 256, n_out, B), dim3(256), 0, st, Gc, pitch, stride, sel, G_out, kcap, n_out,
                     n_keep + m);
  return hipGetLastError();
}

}  // namespace covspec
