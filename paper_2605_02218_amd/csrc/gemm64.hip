// fp64 MFMA GEMM:  C[M,N] (fp64) = A[M,K] * B[N,K]^T (or A * B with B stored [K][N]) with
// A, B stored as fp64, fp32 or bf16 and every product and sum taken in fp64.
//
// Two users.  (1) The fp32-input path: fp32 inputs carry 24-bit mantissas, so an
// fp32-accumulated contraction cannot deliver cosine scores to 1e-5 relative once the cosine
// is small against its natural scale; that workload is small, so its whole chain (embeddings,
// folded query matrix, inner products, norms, Gram matrix) runs on v_mfma_f64_16x16x4_f64 and
// the fp32 storage is the only rounding left.  (2) The low-rank stage, whose block iteration
// on the fp64 Gram matrix is a sequence of fp64 products.
//
// Shape: 256 threads = 4 waves (2x2); wave tile (MI*16) x (NJ*16), block tile twice that in
// each direction (64x64 for <2,2>, 128x128 for <4,4>), k-tile 16.  Operands are converted to
// fp64 on their way into LDS; the loads of k-tile t+1 are issued before the MFMAs of tile t and
// parked in registers, LDS is double buffered, one barrier per k-tile.
// MFMA layouts: operand lane l holds (row|col = l%16, k = l/16); result lane l, register v
// holds (row 4v + l/16, col l%16).
#include <type_traits>
#include "common.h"
#include "host_cache.h"
#include "kernels.h"

namespace covspec {

namespace {

constexpr int TK = 16, PITCH = TK + 1;

__device__ __forceinline__ double as_f64(double v) { return v; }
__device__ __forceinline__ double as_f64(float v) { return (double)v; }
__device__ __forceinline__ double as_f64(bf16_t v) { return (double)bf16_to_f32(v); }

// Workgroups are handed to the 8 XCDs round-robin; regroup the ids so that an XCD works on consecutive
// tiles (same image, same operand rows) and its L2 keeps them.
__device__ __forceinline__ int regroup_xcd(int bid, int nblocks) {
  const int per = nblocks >> 3;
  return (bid < (per << 3)) ? (bid & 7) * per + (bid >> 3) : bid;
}

template <typename TA, typename TB, int EPI, bool GATHER, bool TRANSB, int MI, int NJ>
__global__ __launch_bounds__(256) void gemm64_kernel(GemmArgs g, int tiles_m, int tiles_n) {
  constexpr int TM = 32 * MI, TN = 32 * NJ;
  constexpr int SA = TM / 16, SBn = TN / 16;       // staged elements per thread and operand
  extern __shared__ double smem[];
  double* sA = smem;                               // [2][TM * PITCH]
  double* sB = smem + 2 * TM * PITCH;              // [2][TN * PITCH]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int per = tiles_m * tiles_n;
  const int gid = regroup_xcd(blockIdx.x, gridDim.x);
  const int bidx = gid / per;
  const int pidx = gid - bidx * per;
  const int tm = pidx / tiles_n, tn = pidx - tm * tiles_n;
  const int row0 = tm * TM, col0 = tn * TN;
  const int bo = bidx / g.batch_inner, bi = bidx - bo * g.batch_inner;
  if (g.skip && g.skip[bo] > g.skip_if) return;           // uniform per workgroup
  if (g.lower_only && col0 > row0 + TM - 1) return;       // tile entirely above the diagonal
  const TA* __restrict__ A = (const TA*)g.A + (long)bo * g.strideA + (long)bi * g.strideA2;
  const TB* __restrict__ B = (const TB*)g.B + (long)bo * g.strideB + (long)bi * g.strideB2;
  const long coff = (long)bo * g.strideC + (long)bi * g.strideC2;

  // staging slots.  K-contiguous operand: element e = tid + 256*s -> (row e/16, k e%16).
  // B stored [K][N]: e -> (n = e % TN, k = e / TN), so that a wave reads consecutive n.
  long aoff[SA], boff[SBn];
  bool aok[SA], bok[SBn];
  const int lk = tid & 15;
#pragma unroll
  for (int s = 0; s < SA; ++s) {
    const int ra = row0 + (tid >> 4) + 16 * s;
    aok[s] = ra < g.M;
    long ia = ra;
    if (GATHER && g.gatherA && aok[s]) ia = g.gatherA[(long)bo * g.gstrideA + ra];
    aoff[s] = ia * g.lda + lk;
  }
#pragma unroll
  for (int s = 0; s < SBn; ++s) {
    if (TRANSB) {
      const int e = tid + 256 * s;
      const int n = col0 + (e % TN);
      bok[s] = n < g.N;
      boff[s] = (long)(e / TN) * g.ldb + n;
    } else {
      const int rb = col0 + (tid >> 4) + 16 * s;
      bok[s] = rb < g.N;
      long ib = rb;
      if (GATHER && g.gatherB && bok[s]) ib = g.gatherB[(long)bo * g.gstrideB + rb];
      boff[s] = ib * g.ldb + lk;
    }
  }

  // bf16 x bf16, both K-contiguous, 64 x 64 tiles: a k-tile of an operand is 64 rows x 32 bytes, so the
  // element-wise staging above would issue eight 2-byte loads per thread.  When rows and K allow 16-byte
  // pieces, thread t instead loads ONE piece (operand t / 128, row (t % 128) / 2, half t % 2) and converts its
  // eight values on the way into LDS.
  constexpr bool WIDE_T = std::is_same<TA, bf16_t>::value && std::is_same<TB, bf16_t>::value && !TRANSB && MI == 2 && NJ == 2;
  const bool wide = WIDE_T && g.lda % 8 == 0 && g.ldb % 8 == 0 && g.K % 8 == 0 && (((uintptr_t)A | (uintptr_t)B) & 15) == 0;
  const int wop = tid >> 7, wrow = (tid & 127) >> 1, whalf = tid & 1;
  long woff = 0;
  bool wok = false;
  if (WIDE_T && wide) {
    const int rr = (wop ? col0 : row0) + wrow;
    wok = rr < (wop ? g.N : g.M);
    long ir = rr;
    const int32_t* gl = wop ? g.gatherB : g.gatherA;
    if (GATHER && gl && wok) ir = gl[(long)bo * (wop ? g.gstrideB : g.gstrideA) + rr];
    woff = ir * (wop ? g.ldb : g.lda) + 8 * whalf;
  }
  u32x4_t rw = {0u, 0u, 0u, 0u};

  double ra_[SA], rb_[SBn];
  auto fetch = [&](int k0) {
    if (WIDE_T && wide) {
      const u32x4_t z = {0u, 0u, 0u, 0u};
      const bf16_t* P = wop ? (const bf16_t*)B : (const bf16_t*)A;
      rw = (wok && k0 + 8 * whalf < g.K) ? *(const u32x4_t*)(P + woff + k0) : z;
      return;
    }
#pragma unroll
    for (int s = 0; s < SA; ++s) ra_[s] = (aok[s] && k0 + lk < g.K) ? as_f64(A[aoff[s] + k0]) : 0.0;
#pragma unroll
    for (int s = 0; s < SBn; ++s) {
      if (TRANSB) {
        const int k = k0 + (tid + 256 * s) / TN;
        rb_[s] = (bok[s] && k < g.K) ? as_f64(B[boff[s] + (long)k0 * g.ldb]) : 0.0;
      } else {
        rb_[s] = (bok[s] && k0 + lk < g.K) ? as_f64(B[boff[s] + k0]) : 0.0;
      }
    }
  };
  auto park = [&](int buf) {
    if (WIDE_T && wide) {
      double* dst = (wop ? sB + buf * TN * PITCH : sA + buf * TM * PITCH) + wrow * PITCH + 8 * whalf;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        dst[2 * e] = (double)__uint_as_float(rw[e] << 16);
        dst[2 * e + 1] = (double)__uint_as_float(rw[e] & 0xFFFF0000u);
      }
      return;
    }
    double* a = sA + buf * TM * PITCH;
    double* b = sB + buf * TN * PITCH;
#pragma unroll
    for (int s = 0; s < SA; ++s) a[((tid >> 4) + 16 * s) * PITCH + lk] = ra_[s];
#pragma unroll
    for (int s = 0; s < SBn; ++s) {
      if (TRANSB) {
        const int e = tid + 256 * s;
        b[(e % TN) * PITCH + e / TN] = rb_[s];
      } else {
        b[((tid >> 4) + 16 * s) * PITCH + lk] = rb_[s];
      }
    }
  };

  f64x4_t acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) acc[i][j] = (f64x4_t){0.0, 0.0, 0.0, 0.0};

  const int i16 = lane & 15, kq = lane >> 4;
  const int nt = (g.K + TK - 1) / TK;
  fetch(0);
  park(0);
  __syncthreads();
  for (int t = 0; t < nt; ++t) {
    if (t + 1 < nt) fetch((t + 1) * TK);
    const double* a = sA + (t & 1) * TM * PITCH + (wm * MI * 16 + i16) * PITCH + kq;
    const double* b = sB + (t & 1) * TN * PITCH + (wn * NJ * 16 + i16) * PITCH + kq;
#pragma unroll
    for (int ks = 0; ks < TK / 4; ++ks) {
      double af[MI], bf[NJ];
#pragma unroll
      for (int i = 0; i < MI; ++i) af[i] = a[i * 16 * PITCH + ks * 4];
#pragma unroll
      for (int j = 0; j < NJ; ++j) bf[j] = b[j * 16 * PITCH + ks * 4];
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    if (t + 1 < nt) park((t + 1) & 1);
    __syncthreads();
  }

  if (EPI == EPI_STORE_F64 || EPI == EPI_SUB_F64) {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int r = row0 + wm * MI * 16 + i * 16 + 4 * v + kq;
          const int c = col0 + wn * NJ * 16 + j * 16 + i16;
          if (r < g.M && c < g.N) {
            double* out = (double*)g.C + coff + (long)r * g.ldc + c;
            if (EPI == EPI_SUB_F64) *out -= acc[i][j][v];
            else *out = acc[i][j][v];
            // lanes of equal i16 hold four consecutive rows r: the transposed store goes out in 32-byte pieces
            if (EPI == EPI_STORE_F64 && g.mirror && tn != tm) ((double*)g.C)[coff + (long)c * g.ldc + r] = acc[i][j][v];
          }
        }
  } else {  // EPI_ROWNORM2: per-row sum over this tile's columns of C^2 (fp64)
    double* red = smem;   // [2][TM], reuses the operand buffers (all reads of them are behind the last barrier)
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        double s = 0.0;
#pragma unroll
        for (int j = 0; j < NJ; ++j) s += acc[i][j][v] * acc[i][j][v];
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
        if (i16 == 0) red[wn * TM + wm * MI * 16 + i * 16 + 4 * v + kq] = s;
      }
    __syncthreads();
    if (tid < TM) {
      const int r = row0 + tid;
      if (r < g.M) ((double*)g.C)[coff + (long)r * g.ldc + tn] = red[tid] + red[TM + tid];
    }
  }
}

template <typename TA, typename TB, int EPI, bool GATHER, bool TRANSB, int MI, int NJ>
hipError_t launch_cfg(const GemmArgs& g, hipStream_t stream) {
  constexpr int TM = 32 * MI, TN = 32 * NJ;
  const int tiles_m = (g.M + TM - 1) / TM, tiles_n = (g.N + TN - 1) / TN;
  const long nblocks = (long)tiles_m * tiles_n * g.batch;
  if (nblocks <= 0) return hipSuccess;
  if (nblocks > 0x7fffffffL) return hipErrorInvalidValue;
  const size_t lds = (size_t)2 * (TM + TN) * PITCH * sizeof(double);
  auto kern = gemm64_kernel<TA, TB, EPI, GATHER, TRANSB, MI, NJ>;
  if (lds > 64 * 1024) {
    static PerDeviceInt raised;   // per instantiation
    const hipError_t e = ensure_dynamic_lds(raised, (const void*)kern, lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)nblocks), dim3(256), lds, stream, g, tiles_m, tiles_n);
  return hipGetLastError();
}

// (B stored [K][N] only) 128x128 tiles when they still fill the chip, else 64x64.
inline bool big_tiles(const GemmArgs& g) {
  if (g.M < 128 || g.N < 128) return false;
  const long nb = (long)((g.M + 127) / 128) * ((g.N + 127) / 128) * g.batch;
  return nb >= 256;
}

template <typename TA, typename TB>
hipError_t launch_ab(const GemmArgs& g, hipStream_t stream) {
  const bool gather = g.gatherA || g.gatherB;
  if (g.transB) {
    if (gather) return hipErrorInvalidValue;
    if (g.epilogue == EPI_STORE_F64)
      return big_tiles(g) ? launch_cfg<TA, TB, EPI_STORE_F64, false, true, 4, 4>(g, stream)
                          : launch_cfg<TA, TB, EPI_STORE_F64, false, true, 2, 2>(g, stream);
    if (g.epilogue == EPI_SUB_F64) return launch_cfg<TA, TB, EPI_SUB_F64, false, true, 2, 2>(g, stream);
    return hipErrorInvalidValue;
  }
  if (g.epilogue == EPI_STORE_F64) {
    if (gather) return launch_cfg<TA, TB, EPI_STORE_F64, true, false, 2, 2>(g, stream);
    // 64x64 tiles: measured equal or faster than 128x128 and 128x64 on every workload (the batched products of
    // the low-rank stage make 600-2500 tiles of 128x128, one to two rounds over the device, and the finer tiles
    // lose less to the last, partly filled round than they pay in LDS traffic)
    return launch_cfg<TA, TB, EPI_STORE_F64, false, false, 2, 2>(g, stream);
  }
  if (gather) return hipErrorInvalidValue;
  if (g.epilogue == EPI_SUB_F64) return launch_cfg<TA, TB, EPI_SUB_F64, false, false, 2, 2>(g, stream);
  if (g.epilogue == EPI_ROWNORM2) return launch_cfg<TA, TB, EPI_ROWNORM2, false, false, 2, 2>(g, stream);
  return hipErrorInvalidValue;
}

}  // namespace

int gemm64_tiles_n(int N) { return (N + 63) / 64; }   // ROWNORM2 always runs with 64-column tiles

hipError_t launch_gemm64_bf16(const GemmArgs& g, hipStream_t stream) { return launch_ab<bf16_t, bf16_t>(g, stream); }

hipError_t launch_gemm64_nt(const GemmArgs& g, bool a_is_f64, bool b_is_f64, hipStream_t stream) {
  if (a_is_f64) return b_is_f64 ? launch_ab<double, double>(g, stream) : launch_ab<double, float>(g, stream);
  return b_is_f64 ? launch_ab<float, double>(g, stream) : launch_ab<float, float>(g, stream);
}

}  // namespace covspec
