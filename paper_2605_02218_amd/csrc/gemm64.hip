// fp64 MFMA GEMM for the fp32-input path:  C[M,N] (fp64) = A[M,K] * B[N,K]^T with
// A, B stored as fp32 or fp64 (or both bf16) and every product and sum taken in fp64.
//
// fp32 inputs carry 24-bit mantissas, so an fp32-accumulated contraction cannot
// deliver cosine scores to 1e-5 relative once the cosine is small against its
// natural scale; the fp32 workload is small, so the whole chain (embeddings,
// folded query matrix, inner products, norms, Gram matrix) runs on
// v_mfma_f64_16x16x4_f64 instead and the fp32 storage is the only rounding left.
//
// Shape: 256 threads = 4 waves (2x2), block tile 64x64, wave tile 32x32 = 2x2 MFMA
// tiles, k-tile 16; operands are converted to fp64 while they are staged in LDS.
// MFMA layouts: operand lane l holds (row|col = l%16, k = l/16); result lane l,
// register v holds (row 4v + l/16, col l%16).
#include "common.h"
#include "kernels.h"

namespace covspec {

namespace {

constexpr int TM = 64, TN = 64, TK = 16, PITCH = TK + 1;

__device__ __forceinline__ double as_f64(double v) { return v; }
__device__ __forceinline__ double as_f64(float v) { return (double)v; }
__device__ __forceinline__ double as_f64(bf16_t v) { return (double)bf16_to_f32(v); }

template <typename TA, typename TB, int EPI, bool GATHER, bool TRANSB>
__global__ __launch_bounds__(256) void gemm64_kernel(GemmArgs g, int tiles_m, int tiles_n) {
  __shared__ double sA[TM * PITCH];
  __shared__ double sB[TN * PITCH];
  __shared__ double red[2][TM];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int per = tiles_m * tiles_n;
  const int bidx = blockIdx.x / per;
  const int pidx = blockIdx.x - bidx * per;
  const int tm = pidx / tiles_n, tn = pidx - tm * tiles_n;
  const int row0 = tm * TM, col0 = tn * TN;
  const int bo = bidx / g.batch_inner, bi = bidx - bo * g.batch_inner;
  if (g.skip && g.skip[bo] == g.skip_if) return;   // uniform per workgroup
  const TA* __restrict__ A = (const TA*)g.A + (long)bo * g.strideA + (long)bi * g.strideA2;
  const TB* __restrict__ B = (const TB*)g.B + (long)bo * g.strideB + (long)bi * g.strideB2;
  const long coff = (long)bo * g.strideC + (long)bi * g.strideC2;

  // staging slots: element e = tid + 256*s -> (row e/16, k e%16)
  long aoff[4], boff[4];
  bool aok[4], bok[4];
  const int lk = tid & 15;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int r = (tid >> 4) + 16 * s;
    const int ra = row0 + r, rb = col0 + r;
    aok[s] = ra < g.M;
    bok[s] = rb < g.N;
    long ia = ra, ib = rb;
    if (GATHER) {
      if (g.gatherA && aok[s]) ia = g.gatherA[(long)bo * g.gstrideA + ra];
      if (g.gatherB && bok[s]) ib = g.gatherB[(long)bo * g.gstrideB + rb];
    }
    aoff[s] = ia * g.lda;
    boff[s] = TRANSB ? ib : ib * g.ldb;   // TRANSB: B is stored [K][N], element (n, k) at k*ldb + n
  }

  f64x4_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = (f64x4_t){0.0, 0.0, 0.0, 0.0};

  const int i16 = lane & 15, kq = lane >> 4;
  for (int k0 = 0; k0 < g.K; k0 += TK) {
    const bool kok = k0 + lk < g.K;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int r = (tid >> 4) + 16 * s;
      sA[r * PITCH + lk] = (aok[s] && kok) ? as_f64(A[aoff[s] + k0 + lk]) : 0.0;
      sB[r * PITCH + lk] = (bok[s] && kok) ? as_f64(B[TRANSB ? boff[s] + (long)(k0 + lk) * g.ldb : boff[s] + k0 + lk]) : 0.0;
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < TK / 4; ++ks) {
      double af[2], bf[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        af[i] = sA[(wm * 32 + i * 16 + i16) * PITCH + ks * 4 + kq];
        bf[i] = sB[(wn * 32 + i * 16 + i16) * PITCH + ks * 4 + kq];
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }

  if (EPI == EPI_STORE_F64 || EPI == EPI_SUB_F64) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int r = row0 + wm * 32 + i * 16 + 4 * v + kq;
          const int c = col0 + wn * 32 + j * 16 + i16;
          if (r < g.M && c < g.N) {
            double* out = (double*)g.C + coff + (long)r * g.ldc + c;
            if (EPI == EPI_SUB_F64) *out -= acc[i][j][v];
            else *out = acc[i][j][v];
          }
        }
  } else {  // EPI_ROWNORM2: per-row sum over this tile's columns of C^2 (fp64)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        double s = acc[i][0][v] * acc[i][0][v] + acc[i][1][v] * acc[i][1][v];
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
        if (i16 == 0) red[wn][wm * 32 + i * 16 + 4 * v + kq] = s;
      }
    __syncthreads();
    if (tid < TM) {
      const int r = row0 + tid;
      if (r < g.M) ((double*)g.C)[coff + (long)r * g.ldc + tn] = red[0][tid] + red[1][tid];
    }
  }
}

template <typename TA, typename TB>
hipError_t launch_ab(const GemmArgs& g, hipStream_t stream) {
  const int tiles_m = (g.M + TM - 1) / TM, tiles_n = (g.N + TN - 1) / TN;
  const long nblocks = (long)tiles_m * tiles_n * g.batch;
  if (nblocks <= 0) return hipSuccess;
  if (nblocks > 0x7fffffffL) return hipErrorInvalidValue;
  dim3 grid((unsigned)nblocks), block(256);
  const bool gather = g.gatherA || g.gatherB;
  if (g.transB) {
    if (gather) return hipErrorInvalidValue;
    if (g.epilogue == EPI_STORE_F64) hipLaunchKernelGGL((gemm64_kernel<TA, TB, EPI_STORE_F64, false, true>), grid, block, 0, stream, g, tiles_m, tiles_n);
    else if (g.epilogue == EPI_SUB_F64) hipLaunchKernelGGL((gemm64_kernel<TA, TB, EPI_SUB_F64, false, true>), grid, block, 0, stream, g, tiles_m, tiles_n);
    else return hipErrorInvalidValue;
  } else if (g.epilogue == EPI_STORE_F64) {
    if (gather) hipLaunchKernelGGL((gemm64_kernel<TA, TB, EPI_STORE_F64, true, false>), grid, block, 0, stream, g, tiles_m, tiles_n);
    else hipLaunchKernelGGL((gemm64_kernel<TA, TB, EPI_STORE_F64, false, false>), grid, block, 0, stream, g, tiles_m, tiles_n);
  } else if (g.epilogue == EPI_SUB_F64) {
    hipLaunchKernelGGL((gemm64_kernel<TA, TB, EPI_SUB_F64, false, false>), grid, block, 0, stream, g, tiles_m, tiles_n);
  } else if (g.epilogue == EPI_ROWNORM2) {
    hipLaunchKernelGGL((gemm64_kernel<TA, TB, EPI_ROWNORM2, false, false>), grid, block, 0, stream, g, tiles_m, tiles_n);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace

int gemm64_tiles_n(int N) { return (N + TN - 1) / TN; }

hipError_t launch_gemm64_bf16(const GemmArgs& g, hipStream_t stream) { return launch_ab<bf16_t, bf16_t>(g, stream); }

hipError_t launch_gemm64_nt(const GemmArgs& g, bool a_is_f64, bool b_is_f64, hipStream_t stream) {
  if (a_is_f64) return b_is_f64 ? launch_ab<double, double>(g, stream) : launch_ab<double, float>(g, stream);
  return b_is_f64 ? launch_ab<float, double>(g, stream) : launch_ab<float, float>(g, stream);
}

}  // namespace covspec
