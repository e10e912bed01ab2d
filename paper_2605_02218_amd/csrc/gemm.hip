// MFMA GEMM for gfx950:  C[M,N] = A[M,K] * B[N,K]^T, both operands K-contiguous.
//
// Used for every dense contraction of the token-selection path: the embedding
// projections e(v) = v Wk, e(q) = q Wq (paper Sec. III-A.1), the query/token
// inner products behind the cosine score, and the token Gram matrix of the
// pre-selected tokens behind the rank-r SVD (paper Sec. III-A.3).
//
// Shape: 256 threads = 4 waves in a 2x2 grid, block tile 128x128, wave tile
// 64x64 = 2x2 MFMA 32x32 tiles, k-tile of 128 bytes per row.  Operand tiles go
// global -> registers -> LDS (double buffered, one barrier per k-tile); LDS rows
// are 128 B with the 16-byte chunk index XOR-swizzled by (row & 7), so both the
// 16-byte stores and the MFMA fragment reads are bank-conflict free.
//   bf16: v_mfma_f32_32x32x16_bf16, lane (i = l%32, h = l/32) holds k = 8h..8h+7.
//   fp32: v_mfma_f32_32x32x2_f32; a lane reads two consecutive k and feeds them
//         to two MFMAs (the contraction order is permuted identically for A and B).
// Result layout of both: lane l, register v -> row 8*(v/4) + 4*(l/32) + v%4, col l%32.
#include "common.h"
#include "kernels.h"

namespace covspec {

namespace {

constexpr int BM = 128, BN = 128, ROWB = 128;  // tile rows / cols, bytes per LDS row
constexpr int THREADS = 256;

template <typename In> struct Tr;
template <> struct Tr<bf16_t> { static constexpr int BK = 64; static constexpr int ESZ = 2; };
template <> struct Tr<float> { static constexpr int BK = 32; static constexpr int ESZ = 4; };

__device__ __forceinline__ int swz(int row, int chunk) { return row * ROWB + ((chunk ^ (row & 7)) << 4); }

struct TileMap { int b, tm, tn; };

// 1-D block id -> (batch, tile_m, tile_n).  Consecutive hardware block ids are dealt round-robin
// to the 8 XCDs, so ids are first regrouped to give each XCD (and its private L2) a contiguous
// range of tiles; inside an image, tiles are walked in groups of 8 row-tiles so the group shares
// B tiles while they are L2-resident.
__device__ __forceinline__ TileMap map_block(int bid, int nblocks, int tiles_m, int tiles_n) {
  int v = bid;
  if ((nblocks & 7) == 0) v = (bid & 7) * (nblocks >> 3) + (bid >> 3);
  const int per = tiles_m * tiles_n;
  TileMap t;
  t.b = v / per;
  int p = v - t.b * per;
  constexpr int G = 8;
  int grp = p / (G * tiles_n);
  int first = grp * G;
  int gsz = min(tiles_m - first, G);
  int q = p - grp * G * tiles_n;
  t.tm = first + q % gsz;
  t.tn = q / gsz;
  return t;
}

template <typename In, int EPI, bool GATHER>
__global__ __launch_bounds__(THREADS) void gemm_nt_kernel(GemmArgs g, int tiles_m, int tiles_n) {
  constexpr int BK = Tr<In>::BK;
  constexpr int ESZ = Tr<In>::ESZ;
  constexpr int EPC = 16 / ESZ;  // elements per 16-byte chunk
  __shared__ __attribute__((aligned(16))) unsigned char smem[2][2][BM * ROWB];  // [stage][A|B]

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const TileMap tmap = map_block(blockIdx.x, gridDim.x, tiles_m, tiles_n);
  const int row0 = tmap.tm * BM, col0 = tmap.tn * BN;

  const int bo = tmap.b / g.batch_inner, bi = tmap.b - bo * g.batch_inner;
  const In* __restrict__ A = (const In*)g.A + (long)bo * g.strideA + (long)bi * g.strideA2;
  const In* __restrict__ B = (const In*)g.B + (long)bo * g.strideB + (long)bi * g.strideB2;
  const long coff = (long)bo * g.strideC + (long)bi * g.strideC2;

  // this thread's four (row, chunk) slots of each operand tile
  const int lchunk = tid & 7;
  const int lrow = tid >> 3;  // + 32*s
  long aoff[4], boff[4];
  bool aok[4], bok[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    int ra = row0 + lrow + 32 * s, rb = col0 + lrow + 32 * s;
    aok[s] = ra < g.M;
    bok[s] = rb < g.N;
    long ia = ra, ib = rb;
    if (GATHER) {
      if (g.gatherA && aok[s]) ia = g.gatherA[(long)bo * g.gstrideA + ra];
      if (g.gatherB && bok[s]) ib = g.gatherB[(long)bo * g.gstrideB + rb];
    }
    aoff[s] = ia * g.lda;
    boff[s] = ib * g.ldb;
  }

  u32x4_t ra_[4], rb_[4];
  auto gload = [&](int kt) {
    const int k = kt * BK + lchunk * EPC;
    const bool kok = k < g.K;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      u32x4_t z = {0u, 0u, 0u, 0u};
      ra_[s] = (aok[s] && kok) ? *(const u32x4_t*)(A + aoff[s] + k) : z;
      rb_[s] = (bok[s] && kok) ? *(const u32x4_t*)(B + boff[s] + k) : z;
    }
  };
  auto lstore = [&](int st) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      int r = lrow + 32 * s;
      *(u32x4_t*)(&smem[st][0][swz(r, lchunk)]) = ra_[s];
      *(u32x4_t*)(&smem[st][1][swz(r, lchunk)]) = rb_[s];
    }
  };

  f32x16_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  double acc64[(EPI == EPI_STORE_F64) ? 64 : 1];
  if (EPI == EPI_STORE_F64) {
#pragma unroll
    for (int v = 0; v < 64; ++v) acc64[v] = 0.0;
  }

  const int nk = (g.K + BK - 1) / BK;
  const int li = lane & 31, lh = lane >> 5;
  gload(0);
  lstore(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int st = kt & 1;
    if (kt + 1 < nk) gload(kt + 1);
    const unsigned char* sa = smem[st][0];
    const unsigned char* sb = smem[st][1];
    if constexpr (ESZ == 2) {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        bf16x8_t af[2], bfr[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          int r = wm * 64 + i * 32 + li;
          u32x4_t t = *(const u32x4_t*)(sa + swz(r, 2 * ks + lh));
          af[i] = __builtin_bit_cast(bf16x8_t, t);
          int c = wn * 64 + i * 32 + li;
          u32x4_t u = *(const u32x4_t*)(sb + swz(c, 2 * ks + lh));
          bfr[i] = __builtin_bit_cast(bf16x8_t, u);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int ch = 0; ch < 8; ++ch) {
        float2 af[2], bfr[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          int r = wm * 64 + i * 32 + li;
          af[i] = *(const float2*)(sa + swz(r, ch) + 8 * lh);
          int c = wn * 64 + i * 32 + li;
          bfr[i] = *(const float2*)(sb + swz(c, ch) + 8 * lh);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i].x, bfr[j].x, acc[i][j], 0, 0, 0);
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i].y, bfr[j].y, acc[i][j], 0, 0, 0);
          }
      }
    }
    if (EPI == EPI_STORE_F64) {
      // flush the fp32 partial sums into fp64 every 256 contraction steps
      constexpr int FLUSH = 256 / BK;
      if ((kt % FLUSH) == FLUSH - 1 || kt + 1 == nk) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              acc64[(i * 2 + j) * 16 + v] += (double)acc[i][j][v];
              acc[i][j][v] = 0.f;
            }
      }
    }
    if (kt + 1 < nk) lstore(st ^ 1);
    __syncthreads();
  }

  // ---- epilogue ----
  if (EPI == EPI_STORE_F32 || EPI == EPI_STORE_F64) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          int r = row0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
          int c = col0 + wn * 64 + j * 32 + li;
          if (r < g.M && c < g.N) {
            long o = coff + (long)r * g.ldc + c;
            if (EPI == EPI_STORE_F32) ((float*)g.C)[o] = acc[i][j][v];
            else ((double*)g.C)[o] = acc64[(i * 2 + j) * 16 + v];
          }
        }
  } else if (EPI == EPI_ROWNORM2) {
    // sum over this tile's columns of C^2, one value per row; columns beyond N hold exact zeros
    float* red = (float*)&smem[0][0][0];  // [2][128]
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float s = acc[i][0][v] * acc[i][0][v] + acc[i][1][v] * acc[i][1][v];
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
        if (li == 0) red[wn * 128 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * lh + (v & 3)] = s;
      }
    __syncthreads();
    if (tid < 128) {
      int r = row0 + tid;
      if (r < g.M) ((float*)g.C)[coff + (long)r * g.ldc + tmap.tn] = red[tid] + red[128 + tid];
    }
  }
}

template <typename In, int EPI>
hipError_t launch_t(const GemmArgs& g, hipStream_t stream) {
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  const long nblocks = (long)tiles_m * tiles_n * g.batch;
  if (nblocks <= 0) return hipSuccess;
  if (nblocks > 0x7fffffffL) return hipErrorInvalidValue;
  dim3 grid((unsigned)nblocks), block(THREADS);
  if (g.gatherA || g.gatherB)
    hipLaunchKernelGGL((gemm_nt_kernel<In, EPI, true>), grid, block, 0, stream, g, tiles_m, tiles_n);
  else
    hipLaunchKernelGGL((gemm_nt_kernel<In, EPI, false>), grid, block, 0, stream, g, tiles_m, tiles_n);
  return hipGetLastError();
}

template <typename In>
hipError_t launch_e(const GemmArgs& g, hipStream_t stream) {
  switch (g.epilogue) {
    case EPI_STORE_F32: return launch_t<In, EPI_STORE_F32>(g, stream);
    case EPI_ROWNORM2: return launch_t<In, EPI_ROWNORM2>(g, stream);
    case EPI_STORE_F64: return launch_t<In, EPI_STORE_F64>(g, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

int gemm_tiles_n(int N) { return (N + BN - 1) / BN; }

hipError_t launch_gemm_nt(const GemmArgs& g, int dtype, hipStream_t stream) {
  return dtype == DT_BF16 ? launch_e<bf16_t>(g, stream) : launch_e<float>(g, stream);
}

}  // namespace covspec
