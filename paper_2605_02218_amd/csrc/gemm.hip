// MFMA GEMM for gfx950:  C[M,N] = A[M,K] * B[N,K]^T, both operands K-contiguous.
//
// Used for every dense contraction of the token-selection path: the embedding
// projections e(v) = v Wk, e(q) = q Wq (paper Sec. III-A.1), the query/token
// inner products behind the cosine score, and the token Gram matrix of the
// pre-selected tokens behind the rank-r SVD (paper Sec. III-A.3).
//
// Shape: 256 threads = 4 waves in a 2x2 grid; block tile 128x128 (wave tile 64x64 =
// 2x2 MFMA 32x32 tiles) or, for large problems, 256x256 (wave tile 128x128 = 4x4
// MFMA tiles, 256 accumulator registers); k-tile of 128 bytes per row.  In gemm_nt_kernel operand
// tiles go global -> registers -> LDS (double buffered, one barrier per k-tile); the large bf16
// problems (gemm_nt_ring_kernel) and the gathered fp64-result products (gemm_gram_dma_kernel) load
// straight into LDS.  LDS rows are 128 B with the 16-byte chunk index XOR-swizzled by bits 1-3 of
// the row, so both the 16-byte stores and the MFMA fragment reads are bank-conflict free.
//   bf16: v_mfma_f32_32x32x16_bf16, lane (i = l%32, h = l/32) holds k = 8h..8h+7.
//   fp32: v_mfma_f32_32x32x2_f32; a lane reads two consecutive k and feeds them
//         to two MFMAs (the contraction order is permuted identically for A and B).
// Result layout of both: lane l, register v -> row 8*(v/4) + 4*(l/32) + v%4, col l%32.
#include <type_traits>

#include "common.h"
#include "host_cache.h"
#include "kernels.h"

namespace covspec {

namespace {

constexpr int ROWB = 128;  // bytes per LDS row (one k-tile of a tile row)
constexpr int THREADS = 256;

template <typename In> struct Tr;
template <> struct Tr<bf16_t> { static constexpr int BK = 64; static constexpr int ESZ = 2; };
template <> struct Tr<float> { static constexpr int BK = 32; static constexpr int ESZ = 4; };

// Two 128-byte rows fill the 64 banks once, so rows of equal parity share their banks: the 16-byte chunk index is
// XORed with bits 1-3 of the row, which puts any 16 consecutive rows' chunk c on 16 distinct bank groups (one
// ds_read_b128 of 16 lanes is then free of conflicts; with bits 0-2 as the key rows r and r + 8 collided, and the
// bank-conflict counter read more conflict cycles than active ones).  8-byte reads of 32 consecutive rows (the
// fp32 path) additionally swap the two halves of a chunk in rows with bit 4 set: swz_half.
__device__ __forceinline__ int swz(int row, int chunk) { return row * ROWB + ((chunk ^ ((row >> 1) & 7)) << 4); }
__device__ __forceinline__ int swz_half(int row) { return (row & 16) >> 1; }   // 0 or 8 bytes

// 64-byte LDS rows (a k-tile of 32 bf16, the Gram kernel): 4 chunks, chunk index XORed with bit2(row) |
// (bit1(row)^bit3(row))<<1, which keeps every aligned group of 8 and of 16 consecutive rows on distinct banks for
// 16-byte reads.
__device__ __forceinline__ int swz64(int row, int chunk) {
  const int f = ((row >> 2) & 1) | ((((row >> 1) ^ (row >> 3)) & 1) << 1);
  return row * 64 + ((chunk ^ f) << 4);
}

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

// TW = MFMA 32x32 tiles per wave and dimension: block tile (64*TW)^2, wave tile (32*TW)^2.
template <typename In, int EPI, bool GATHER, int TW>
__global__ __launch_bounds__(THREADS) void gemm_nt_kernel(GemmArgs g, int tiles_m, int tiles_n) {
  constexpr int BK = Tr<In>::BK;
  constexpr int ESZ = Tr<In>::ESZ;
  constexpr int EPC = 16 / ESZ;       // elements per 16-byte chunk
  constexpr int BT = 64 * TW;         // block tile rows = cols
  constexpr int WT = 32 * TW;         // wave tile rows = cols
  constexpr int NS = BT / 32;         // 16-byte load slots per thread and operand
  constexpr int STAGE = 2 * BT * ROWB;  // bytes per stage: A tile then B tile
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // [2][A|B][BT*ROWB]

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const TileMap tmap = map_block(blockIdx.x, gridDim.x, tiles_m, tiles_n);
  const int row0 = tmap.tm * BT, col0 = tmap.tn * BT;
  if (g.lower_only && tmap.tn > tmap.tm) return;      // square tiles: entirely above the diagonal (uniform)

  const int bo = tmap.b / g.batch_inner, bi = tmap.b - bo * g.batch_inner;
  const In* __restrict__ A = (const In*)g.A + (long)bo * g.strideA + (long)bi * g.strideA2;
  const In* __restrict__ B = (const In*)g.B + (long)bo * g.strideB + (long)bi * g.strideB2;
  const long coff = (long)bo * g.strideC + (long)bi * g.strideC2;

  // this thread's (row, chunk) slots of each operand tile: rows lrow + 32*s, chunk lchunk.  Without a
  // gather list the slots are a fixed stride apart, so one base offset per operand is kept.
  const int lchunk = tid & 7;
  const int lrow = tid >> 3;
  long aoff[GATHER ? NS : 1], boff[GATHER ? NS : 1];
  if (GATHER) {
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int ra = row0 + lrow + 32 * s, rb = col0 + lrow + 32 * s;
      long ia = ra, ib = rb;
      if (g.gatherA && ra < g.M) ia = g.gatherA[(long)bo * g.gstrideA + ra];
      if (g.gatherB && rb < g.N) ib = g.gatherB[(long)bo * g.gstrideB + rb];
      aoff[GATHER ? s : 0] = ia * g.lda;
      boff[GATHER ? s : 0] = ib * g.ldb;
    }
  } else {
    aoff[0] = (long)(row0 + lrow) * g.lda;
    boff[0] = (long)(col0 + lrow) * g.ldb;
  }
  const long astep = 32 * g.lda, bstep = 32 * g.ldb;
  const int arows = g.M - row0 - lrow, brows = g.N - col0 - lrow;   // slot s is in range iff 32*s < rows

  // global -> registers -> LDS staging of the next k-tile (a second register set, to give loads two
  // k-tiles to land, was measured slower: the extra registers and moves cost more than the latency hid)
  u32x4_t ra0[NS], rb0[NS];
  auto gload = [&](int kt, u32x4_t (&ra_)[NS], u32x4_t (&rb_)[NS]) {
    const int k = kt * BK + lchunk * EPC;
    const bool kok = k < g.K;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      u32x4_t z = {0u, 0u, 0u, 0u};
      const long ao = GATHER ? aoff[GATHER ? s : 0] : aoff[0] + s * astep;
      const long bo_ = GATHER ? boff[GATHER ? s : 0] : boff[0] + s * bstep;
      ra_[s] = (32 * s < arows && kok) ? *(const u32x4_t*)(A + ao + k) : z;
      rb_[s] = (32 * s < brows && kok) ? *(const u32x4_t*)(B + bo_ + k) : z;
    }
  };
  auto lstore = [&](int st, const u32x4_t (&ra_)[NS], const u32x4_t (&rb_)[NS]) {
    unsigned char* sa = smem + st * STAGE;
    unsigned char* sb = sa + BT * ROWB;
    const bool flip = ESZ == 4 && (lrow & 16);     // fp32: rows with bit 4 set keep the halves of a chunk swapped
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      int r = lrow + 32 * s;
      const u32x4_t va = ra_[s], vb = rb_[s];
      *(u32x4_t*)(sa + swz(r, lchunk)) = flip ? (u32x4_t){va[2], va[3], va[0], va[1]} : va;
      *(u32x4_t*)(sb + swz(r, lchunk)) = flip ? (u32x4_t){vb[2], vb[3], vb[0], vb[1]} : vb;
    }
  };

  f32x16_t acc[TW][TW];
#pragma unroll
  for (int i = 0; i < TW; ++i)
#pragma unroll
    for (int j = 0; j < TW; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  double acc64[(EPI == EPI_STORE_F64) ? TW * TW * 16 : 1];
  if (EPI == EPI_STORE_F64) {
#pragma unroll
    for (int v = 0; v < TW * TW * 16; ++v) acc64[v] = 0.0;
  }

  const int nk = (g.K + BK - 1) / BK;
  const int li = lane & 31, lh = lane >> 5;

  auto compute = [&](int st) {
    const unsigned char* sa = smem + st * STAGE;
    const unsigned char* sb = sa + BT * ROWB;
    if constexpr (ESZ == 2) {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        bf16x8_t af[TW], bfr[TW];
#pragma unroll
        for (int i = 0; i < TW; ++i) {
          int r = wm * WT + i * 32 + li;
          u32x4_t t = *(const u32x4_t*)(sa + swz(r, 2 * ks + lh));
          af[i] = __builtin_bit_cast(bf16x8_t, t);
          int c = wn * WT + i * 32 + li;
          u32x4_t u = *(const u32x4_t*)(sb + swz(c, 2 * ks + lh));
          bfr[i] = __builtin_bit_cast(bf16x8_t, u);
        }
#pragma unroll
        for (int i = 0; i < TW; ++i)
#pragma unroll
          for (int j = 0; j < TW; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int ch = 0; ch < 8; ++ch) {
        float2 af[TW], bfr[TW];
#pragma unroll
        for (int i = 0; i < TW; ++i) {
          int r = wm * WT + i * 32 + li;
          af[i] = *(const float2*)(sa + swz(r, ch) + ((8 * lh) ^ swz_half(r)));
          int c = wn * WT + i * 32 + li;
          bfr[i] = *(const float2*)(sb + swz(c, ch) + ((8 * lh) ^ swz_half(c)));
        }
#pragma unroll
        for (int i = 0; i < TW; ++i)
#pragma unroll
          for (int j = 0; j < TW; ++j) {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i].x, bfr[j].x, acc[i][j], 0, 0, 0);
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i].y, bfr[j].y, acc[i][j], 0, 0, 0);
          }
      }
    }
  };
  auto flush64 = [&](int kt) {
    if (EPI == EPI_STORE_F64) {
      // flush the fp32 partial sums into fp64 every 256 contraction steps
      constexpr int FLUSH = 256 / BK;
      if ((kt % FLUSH) == FLUSH - 1 || kt + 1 == nk) {
#pragma unroll
        for (int i = 0; i < TW; ++i)
#pragma unroll
          for (int j = 0; j < TW; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              acc64[(i * TW + j) * 16 + v] += (double)acc[i][j][v];
              acc[i][j][v] = 0.f;
            }
      }
    }
  };

  gload(0, ra0, rb0);
  lstore(0, ra0, rb0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int st = kt & 1;
    if (kt + 1 < nk) gload(kt + 1, ra0, rb0);   // lands while this k-tile feeds the MFMAs
    compute(st);
    flush64(kt);
    if (kt + 1 < nk) lstore(st ^ 1, ra0, rb0);
    __syncthreads();
  }

  // ---- epilogue ----
  if (EPI == EPI_STORE_F32 || EPI == EPI_STORE_F64) {
#pragma unroll
    for (int i = 0; i < TW; ++i)
#pragma unroll
      for (int j = 0; j < TW; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          int r = row0 + wm * WT + i * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
          int c = col0 + wn * WT + j * 32 + li;
          if (r < g.M && c < g.N) {
            long o = coff + (long)r * g.ldc + c;
            if (EPI == EPI_STORE_F32) ((float*)g.C)[o] = acc[i][j][v];
            else {
              ((double*)g.C)[o] = acc64[(i * TW + j) * 16 + v];
              // symmetric product: the tile below the diagonal is also stored transposed (v & 3 walks four
              // consecutive rows r, so each thread writes 32 contiguous bytes of row c)
              if (g.mirror && tmap.tn != tmap.tm) ((double*)g.C)[coff + (long)c * g.ldc + r] = acc64[(i * TW + j) * 16 + v];
            }
          }
        }
  } else if (EPI == EPI_ROWNORM2) {
    // per row: sum over 128 output columns of C^2 (columns beyond N hold exact zeros).  A wave covers WT
    // columns: with TW = 2 the two wave columns are combined through LDS, with TW = 4 each wave column is
    // one 128-column part of its own.
    float* red = (float*)smem;  // [2][BT]
#pragma unroll
    for (int i = 0; i < TW; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < TW; ++j) s = fmaf(acc[i][j][v], acc[i][j][v], s);
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
        if (li == 0) red[wn * BT + wm * WT + i * 32 + 8 * (v >> 2) + 4 * lh + (v & 3)] = s;
      }
    __syncthreads();
    for (int t = tid; t < BT; t += THREADS) {
      int r = row0 + t;
      if (r < g.M) {
        float* out = (float*)g.C + coff + (long)r * g.ldc;
        if (TW == 2) out[tmap.tn] = red[t] + red[BT + t];
        else {
          out[2 * tmap.tn] = red[t];
          if ((2 * tmap.tn + 1) * 128 < g.N) out[2 * tmap.tn + 1] = red[BT + t];
        }
      }
    }
  }
}

template <int EPI>
__device__ __forceinline__ void dma_epilogue(f32x16_t (&acc)[4][4], const GemmArgs& g, long coff, int row0, int col0, int tn,
                                             unsigned char* smem) {
  constexpr int BT = 256, WT = 128, TW = 4;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int li = lane & 31, lh = lane >> 5;
  if (EPI == EPI_STORE_F32) {
#pragma unroll
    for (int i = 0; i < TW; ++i)
#pragma unroll
      for (int j = 0; j < TW; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          int r = row0 + wm * WT + i * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
          int c = col0 + wn * WT + j * 32 + li;
          if (r < g.M && c < g.N) ((float*)g.C)[coff + (long)r * g.ldc + c] = acc[i][j][v];
        }
  } else {
    // EPI_ROWNORM2: one part per wave column (128 output columns), so a wave reduces its own 128 x 128 tile: every
    // lane adds its four column groups, puts its 64 partial sums into the wave's own LDS block as [lane column]
    // [row] (pitch 132 floats: the 16-byte stores of 16 lanes and the 4-byte reads of 64 lanes fall on distinct
    // banks), and then lane t adds the 32 lane columns of rows t and t + 64.  (Butterfly shuffles, five per value,
    // took 16 us per tile.)
    constexpr int PITCH = WT + 4;
    float* wbuf = (float*)smem + wave * (32 * PITCH);
#pragma unroll
    for (int i = 0; i < TW; ++i)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        f32x4_t s4;
#pragma unroll
        for (int vr = 0; vr < 4; ++vr) {
          float s = 0.f;
#pragma unroll
          for (int j = 0; j < TW; ++j)
            if (col0 + wn * WT + j * 32 + li < g.N) s = fmaf(acc[i][j][4 * vq + vr], acc[i][j][4 * vq + vr], s);
          s4[vr] = s;
        }
        *(f32x4_t*)(wbuf + li * PITCH + i * 32 + 8 * vq + 4 * lh) = s4;
      }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the wave's own stores are in LDS before its lanes read them
    const int part = 2 * tn + wn;
    if (part * 128 < g.N) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int rr = lane + 64 * h;
        float s = 0.f;
#pragma unroll
        for (int l = 0; l < 32; ++l) s += wbuf[l * PITCH + rr];
        const int r = row0 + wm * WT + rr;
        if (r < g.M) ((float*)g.C)[coff + (long)r * g.ldc + part] = s;
      }
    }
  }
}

// ---- large bf16 problems: 256x256 block tile (four waves as 2x2, wave tile 128x128 = 4x4 MFMA tiles, 256
// accumulator registers), k-tiles of 64 (K % 64 == 0, K >= 128) and a ring of operand tiles in LDS.
// Loads: every direct-to-LDS load covers whole 128-byte lines of 8 rows (the vector L1 streams whole lines at 33 TB/s
// from L2-resident data, 64-byte halves at 18 TB/s; the tile needs 20 TB/s at the full MFMA rate).  They are buffer
// loads: the operand of the output tile's image is a raw buffer (base in scalar registers, range = its bytes, so a
// row beyond M / N loads zeros instead of faulting), a lane's row and chunk are a 32-bit offset that never changes,
// and the tile row and the k-tile are the instruction's scalar offset: a load is one instruction with no vector
// arithmetic in front of it.
// Ring: the four SIMDs of a compute unit share one address unit that takes 16 cycles per 1 KB load, 1024 cycles per
// k-tile against 2048 cycles of MFMAs; loads that all go out in one quarter of the k-tile (as two whole stages force;
// measured: that quarter took 1550 cycles instead of 512 and the kernel stayed at 0.43 of the peak) stall their waves
// at issue.  So the 160 KB of LDS are a ring of five 32 KB slots that hold operand tiles in the order A0 B0 A1 B1
// A2 ...: while k-tile T is multiplied, A(T+1) is resident and B(T+1) half resident, and every k-step (16 MFMAs per
// wave) issues one quarter of a k-tile's loads (4 per wave, one per two MFMAs of its second half): the second half of
// B(T+1), the two halves of A(T+2) into the fifth slot, the first half of B(T+2) into the slot A(T) has just left.
// One barrier per k-tile, after the fragments of its fourth k-step are in registers: tile T+1 has landed (at most
// the 8 loads of A(T+2) are outstanding) and T's slots are free.
template <int EPI>
__global__ __launch_bounds__(THREADS) void gemm_nt_ring_kernel(GemmArgs g, int tiles_m, int tiles_n) {
  constexpr int BT = 256, WT = 128, TW = 4, BK = 64;
  constexpr int SLOT = BT * ROWB;     // bytes of one operand tile
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // [5][SLOT]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int wm = wave >> 1, wn = wave & 1;
  const int li = lane & 31, lh = lane >> 5;
  const int nk = g.K / BK;
  const TileMap tmap = map_block(blockIdx.x, gridDim.x, tiles_m, tiles_n);
  const int row0 = tmap.tm * BT, col0 = tmap.tn * BT;
  const int bo = tmap.b / g.batch_inner, bi = tmap.b - bo * g.batch_inner;
  const bf16_t* __restrict__ A = (const bf16_t*)g.A + (long)bo * g.strideA + (long)bi * g.strideA2;
  const bf16_t* __restrict__ B = (const bf16_t*)g.B + (long)bo * g.strideB + (long)bi * g.strideB2;
  const long coff = (long)bo * g.strideC + (long)bi * g.strideC2;
  auto m5 = [](int x) { return x >= 5 ? x - 5 : x; };

  // Wave w issues loads j = 0..7 per operand tile; load j fills tile rows 8*(8w+j) .. +7: lane l -> row
  // 8*(8w+j) + l/8, physical chunk l%8, which holds logical chunk (l%8) ^ bits 1-3 of the row = (l%8) ^
  // (4 (j & 1) + l/16).  A lane's byte offset inside the image is v[j & 1] + (tile row 0 + 8 j) * pitch; the second
  // term and the k-tile go into the instruction's scalar offset.
  const int pitchA = g.lda * 2, pitchB = g.ldb * 2;
  const int rl = 64 * wave + (lane >> 3);
  int va[2], vb[2];
#pragma unroll
  for (int par = 0; par < 2; ++par) {
    const int c = (lane & 7) ^ (4 * par + (lane >> 4));
    va[par] = rl * pitchA + c * 16;
    vb[par] = rl * pitchB + c * 16;
  }
  const __amdgpu_buffer_rsrc_t rsrcA =
      __builtin_amdgcn_make_buffer_rsrc((void*)A, (short)0, (int)(((long)(g.M - 1) * g.lda + g.K) * 2), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcB =
      __builtin_amdgcn_make_buffer_rsrc((void*)B, (short)0, (int)(((long)(g.N - 1) * g.ldb + g.K) * 2), 0x00020000);
  const int sa0 = row0 * pitchA, sb0 = col0 * pitchB;
  // load j (0..7) of this wave for operand tile A / B of k-tile lkt into a slot
  auto load_one = [&](bool opB, int j, int slot, int lkt) {
    unsigned char* dst = smem + slot * SLOT + wave_u * 8192 + j * 1024;
    const int so = lkt * (BK * 2) + (opB ? sb0 : sa0) + j * 8 * (opB ? pitchB : pitchA);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(opB ? rsrcB : rsrcA, (__attribute__((address_space(3))) void*)dst, 16,
                                             opB ? vb[j & 1] : va[j & 1], so, 0, 0);
  };
  auto load_half = [&](bool opB, int half, int slot, int lkt) {
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) load_one(opB, 4 * half + jj, slot, lkt);
  };

  f32x16_t acc[TW][TW];
#pragma unroll
  for (int i = 0; i < TW; ++i)
#pragma unroll
    for (int j = 0; j < TW; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  // fragment byte offsets inside an operand tile per k-step; the 32-row groups of a wave are 4096 bytes apart (the
  // swizzle key repeats every 16 rows)
  int offA[4], offB[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    offA[ks] = swz(wm * WT + li, 2 * ks + lh);
    offB[ks] = swz(wn * WT + li, 2 * ks + lh);
  }
  auto frags = [&](int slotA, int slotB, int ks, bf16x8_t (&af)[TW], bf16x8_t (&bfr)[TW]) {
    const unsigned char* pa = smem + slotA * SLOT + offA[ks];
    const unsigned char* pb = smem + slotB * SLOT + offB[ks];
#pragma unroll
    for (int i = 0; i < TW; ++i) {
      af[i] = __builtin_bit_cast(bf16x8_t, *(const u32x4_t*)(pa + i * 32 * ROWB));
      bfr[i] = __builtin_bit_cast(bf16x8_t, *(const u32x4_t*)(pb + i * 32 * ROWB));
    }
  };
  auto mma = [&](const bf16x8_t (&af)[TW], const bf16x8_t (&bfr)[TW]) {
#pragma unroll
    for (int i = 0; i < TW; ++i)
#pragma unroll
      for (int j = 0; j < TW; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
  };
  // One k-step: the fragments of the next k-step (slots sa / sb, k-step ks) into the idle register set, one quarter
  // of an operand tile's loads, the 16 MFMAs of this k-step.  The source is written in the order in which the
  // instructions are to go out (a load into LDS is not moved across a read of LDS by the compiler), and scheduling
  // groups spread them: per four MFMAs two fragment reads and one load, so that the LDS sees the reads of the four
  // waves evenly (all eight in the first half of the k-step keep it busy all of that half, and a read that cannot be
  // queued holds up the MFMA behind it).  Read order a0 b0 | b1 b2 | b3 a1 | a2 a3: every fragment is in its
  // register at least eight MFMAs before the first MFMA that needs it.
  auto kstep = [&](int sa, int sb, int ks, bf16x8_t (&af)[TW], bf16x8_t (&bfr)[TW], const bf16x8_t (&ca)[TW], const bf16x8_t (&cb)[TW],
                   bool opB, int half, int slot, int lkt) {
    const unsigned char* pa = smem + sa * SLOT + offA[ks];
    const unsigned char* pb = smem + sb * SLOT + offB[ks];
    auto ra = [&](int i) { af[i] = __builtin_bit_cast(bf16x8_t, *(const u32x4_t*)(pa + i * 32 * ROWB)); };
    auto rb = [&](int i) { bfr[i] = __builtin_bit_cast(bf16x8_t, *(const u32x4_t*)(pb + i * 32 * ROWB)); };
    ra(0); rb(0);
    load_one(opB, 4 * half + 0, slot, lkt);
    rb(1); rb(2);
    load_one(opB, 4 * half + 1, slot, lkt);
    rb(3); ra(1);
    load_one(opB, 4 * half + 2, slot, lkt);
    ra(2); ra(3);
    load_one(opB, 4 * half + 3, slot, lkt);
    mma(ca, cb);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // DS read
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // VMEM read (global -> LDS)
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    }
  };

  load_half(false, 0, 0, 0);
  load_half(false, 1, 0, 0);
  load_half(true, 0, 1, 0);
  load_half(true, 1, 1, 0);
  load_half(false, 0, 2, 1);
  load_half(false, 1, 2, 1);
  load_half(true, 0, 3, 1);
  __builtin_amdgcn_s_waitcnt(0x007c);   // vmcnt(12) lgkmcnt(0): k-tile 0 has landed
  __builtin_amdgcn_s_barrier();
  bf16x8_t a0[TW], b0[TW], a1[TW], b1[TW];
  frags(0, 1, 0, a0, b0);
  int ua = 0;   // slot of A of the k-tile being multiplied; B follows it, then A and B of the next k-tile, then A(T+2)
  // The body is branch-free: past the end the loads repeat the last k-tile into slots nobody reads any more and the
  // fourth k-step reads fragments that are never used.
  for (int kt = 0; kt < nk; ++kt) {
    const int sA = ua, sB = m5(ua + 1), sA1 = m5(ua + 2), sB1 = m5(ua + 3), sA2 = m5(ua + 4);
    const int k1 = min(kt + 1, nk - 1), k2 = min(kt + 2, nk - 1);
    __builtin_amdgcn_sched_barrier(0);
    kstep(sA, sB, 1, a1, b1, a0, b0, true, 1, sB1, k1);
    __builtin_amdgcn_sched_barrier(0);
    kstep(sA, sB, 2, a0, b0, a1, b1, false, 0, sA2, k2);
    __builtin_amdgcn_sched_barrier(0);
    kstep(sA, sB, 3, a1, b1, a0, b0, false, 1, sA2, k2);
    __builtin_amdgcn_sched_barrier(0);
    // k-tile T+1 has landed in every wave's share and every wave has read its last fragments of k-tile T
    __builtin_amdgcn_s_waitcnt(0x0078);   // vmcnt(8) lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    kstep(sA1, sB1, 0, a0, b0, a1, b1, true, 0, sA, k2);
    __builtin_amdgcn_sched_barrier(0);
    ua = sA1;
  }
  __builtin_amdgcn_s_waitcnt(0x0070);
  __builtin_amdgcn_s_barrier();
  dma_epilogue<EPI>(acc, g, coff, row0, col0, tmap.tn, smem);
}

template <int EPI>
hipError_t launch_ring(const GemmArgs& g, hipStream_t stream) {
  constexpr int BT = 256, LDS = 5 * BT * ROWB;
  const int tiles_m = (g.M + BT - 1) / BT, tiles_n = (g.N + BT - 1) / BT;
  const long nblocks = (long)tiles_m * tiles_n * g.batch;
  if (nblocks > 0x7fffffffL) return hipErrorInvalidValue;
  auto kern = gemm_nt_ring_kernel<EPI>;
  static PerDeviceInt raised;   // per instantiation
  const hipError_t attr = ensure_dynamic_lds(raised, (const void*)kern, LDS);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(kern, dim3((unsigned)nblocks), dim3(THREADS), LDS, stream, g, tiles_m, tiles_n);
  return hipGetLastError();
}

// ---- bf16 products into fp64 with optional row gathers (the Gram matrix of the pre-selected tokens and the rows a
// streaming step adds to it): 128x128 block tile, wave tile 64x64 (2x2 MFMA tiles), k-tile 32, four LDS stages of
// 16 KB filled by direct global -> LDS loads whose lanes take their row from the gather list, fp32 partial sums
// flushed into fp64 accumulators every 256 k, tiles above the diagonal skipped and mirrored on request.  One barrier
// per k-tile, the fragments of the next k-tile read while the current one is multiplied; two workgroups fit a compute unit, so one's waits are the other's MFMAs.  Rows beyond M / N are
// clamped when loading and masked in the epilogue; requires K % 32 == 0.
__global__ __launch_bounds__(THREADS, 2) void gemm_gram_dma_kernel(GemmArgs g, int tiles_m, int tiles_n) {
  constexpr int BT = 128, WT = 64, TW = 2, BK = 32, NST = 4;
  constexpr int STAGE = 2 * BT * 64;  // bytes: A tile then B tile
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const TileMap tmap = map_block(blockIdx.x, gridDim.x, tiles_m, tiles_n);
  if (g.lower_only && tmap.tn > tmap.tm) return;      // square tiles: entirely above the diagonal (uniform)
  const int row0 = tmap.tm * BT, col0 = tmap.tn * BT;
  const int bo = tmap.b / g.batch_inner, bi = tmap.b - bo * g.batch_inner;
  const bf16_t* __restrict__ A = (const bf16_t*)g.A + (long)bo * g.strideA + (long)bi * g.strideA2;
  const bf16_t* __restrict__ B = (const bf16_t*)g.B + (long)bo * g.strideB + (long)bi * g.strideB2;
  const long coff = (long)bo * g.strideC + (long)bi * g.strideC2;

  // wave w issues loads j = 0, 1 per operand and stage; load j fills tile rows 16*(2w+j) .. +15:
  // lane l -> row 16*(2w+j) + l/4, physical chunk l%4
  const bf16_t* ga[2];
  const bf16_t* gb[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int r = 16 * (2 * wave + j) + (lane >> 2);
    const int f = ((r >> 2) & 1) | ((((r >> 1) ^ (r >> 3)) & 1) << 1);
    const int c = (lane & 3) ^ f;  // logical chunk that belongs at this physical slot
    long ra = min(row0 + r, g.M - 1), rb = min(col0 + r, g.N - 1);
    if (g.gatherA) ra = g.gatherA[(long)bo * g.gstrideA + ra];
    if (g.gatherB) rb = g.gatherB[(long)bo * g.gstrideB + rb];
    ga[j] = A + ra * g.lda + c * 8;
    gb[j] = B + rb * g.ldb + c * 8;
  }
  auto issue = [&](int kt) {
    unsigned char* sa = smem + (kt & (NST - 1)) * STAGE + wave * 2048;
    unsigned char* sb = sa + BT * 64;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(ga[j] + kt * BK),
                                       (__attribute__((address_space(3))) void*)(sa + j * 1024), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gb[j] + kt * BK),
                                       (__attribute__((address_space(3))) void*)(sb + j * 1024), 16, 0, 0);
    }
  };

  f32x16_t acc[TW][TW];
  double acc64[TW * TW * 16];
#pragma unroll
  for (int i = 0; i < TW; ++i)
#pragma unroll
    for (int j = 0; j < TW; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) { acc[i][j][v] = 0.f; acc64[(i * TW + j) * 16 + v] = 0.0; }

  const int nk = g.K / BK;
  const int li = lane & 31, lh = lane >> 5;
  int offA[2][TW], offB[2][TW];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks)
#pragma unroll
    for (int i = 0; i < TW; ++i) {
      offA[ks][i] = swz64(wm * WT + i * 32 + li, 2 * ks + lh);
      offB[ks][i] = BT * 64 + swz64(wn * WT + i * 32 + li, 2 * ks + lh);
    }
  auto frags = [&](const unsigned char* st, int ks, bf16x8_t (&af)[TW], bf16x8_t (&bfr)[TW]) {
#pragma unroll
    for (int i = 0; i < TW; ++i) {
      af[i] = __builtin_bit_cast(bf16x8_t, *(const u32x4_t*)(st + offA[ks][i]));
      bfr[i] = __builtin_bit_cast(bf16x8_t, *(const u32x4_t*)(st + offB[ks][i]));
    }
  };
  auto mma = [&](const bf16x8_t (&af)[TW], const bf16x8_t (&bfr)[TW]) {
#pragma unroll
    for (int i = 0; i < TW; ++i)
#pragma unroll
      for (int j = 0; j < TW; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
  };
  auto flush = [&]() {
#pragma unroll
    for (int i = 0; i < TW; ++i)
#pragma unroll
      for (int j = 0; j < TW; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          acc64[(i * TW + j) * 16 + v] += (double)acc[i][j][v];
          acc[i][j][v] = 0.f;
        }
  };
  auto stage_ptr = [&](int kt) -> const unsigned char* { return smem + (kt & (NST - 1)) * STAGE; };

  // Per k-tile kt: wait until tile kt+1 has landed (only the four loads of tile kt+2 may be outstanding), barrier,
  // start the loads of tile kt+3 into the stage that held tile kt-1 (every wave has read it: its LDS reads are
  // complete before it arrives at the barrier).  The fragments are prefetched one k-step ahead, in two register
  // sets: the second k-step of tile kt is read while the first one feeds the MFMAs, the first k-step of tile
  // kt+1 while the second one does.  Past the end, `issue` re-loads the last tile and `frags` reads a stage whose
  // values are never used.
  bf16x8_t a0[TW], b0[TW], a1[TW], b1[TW];
  issue(0);
  issue(min(1, nk - 1));
  issue(min(2, nk - 1));
  __builtin_amdgcn_s_waitcnt(0x0078);   // vmcnt(8) lgkmcnt(0): tile 0 has landed
  __builtin_amdgcn_s_barrier();
  frags(stage_ptr(0), 0, a0, b0);
  for (int kt = 0; kt < nk; ++kt) {
    __builtin_amdgcn_s_waitcnt(0x0074);   // vmcnt(4) lgkmcnt(0): all but the newest tile have landed
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    frags(stage_ptr(kt), 1, a1, b1);
    issue(min(kt + 3, nk - 1));
    mma(a0, b0);
    __builtin_amdgcn_sched_barrier(0);
    frags(stage_ptr(kt + 1), 0, a0, b0);
    mma(a1, b1);
    __builtin_amdgcn_sched_barrier(0);
    // the fp32 partial sums go into fp64 every 256 contraction steps (8 k-tiles) and at the end
    if ((kt & 7) == 7 || kt + 1 == nk) flush();
  }
  __builtin_amdgcn_s_waitcnt(0x0070);

#pragma unroll
  for (int i = 0; i < TW; ++i)
#pragma unroll
    for (int j = 0; j < TW; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int r = row0 + wm * WT + i * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
        const int c = col0 + wn * WT + j * 32 + li;
        if (r < g.M && c < g.N) {
          const double x = acc64[(i * TW + j) * 16 + v];
          ((double*)g.C)[coff + (long)r * g.ldc + c] = x;
          // symmetric product: the tile below the diagonal is also stored transposed (v & 3 walks four
          // consecutive rows r, so each thread writes 32 contiguous bytes of row c)
          if (g.mirror && tmap.tn != tmap.tm) ((double*)g.C)[coff + (long)c * g.ldc + r] = x;
        }
      }
}

inline hipError_t launch_gram_dma(const GemmArgs& g, hipStream_t stream) {
  constexpr int BT = 128, LDS = 4 * 2 * BT * 64;
  const int tiles_m = (g.M + BT - 1) / BT, tiles_n = (g.N + BT - 1) / BT;
  const long nblocks = (long)tiles_m * tiles_n * g.batch;
  if (nblocks <= 0) return hipSuccess;
  if (nblocks > 0x7fffffffL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(gemm_gram_dma_kernel, dim3((unsigned)nblocks), dim3(THREADS), LDS, stream, g, tiles_m, tiles_n);
  return hipGetLastError();
}

template <typename In, int EPI, bool GATHER, int TW>
hipError_t launch_cfg(const GemmArgs& g, hipStream_t stream) {
  constexpr int BT = 64 * TW;
  constexpr int LDS = 2 * 2 * BT * ROWB;
  const int tiles_m = (g.M + BT - 1) / BT, tiles_n = (g.N + BT - 1) / BT;
  const long nblocks = (long)tiles_m * tiles_n * g.batch;
  if (nblocks <= 0) return hipSuccess;
  if (nblocks > 0x7fffffffL) return hipErrorInvalidValue;
  auto kern = gemm_nt_kernel<In, EPI, GATHER, TW>;
  static PerDeviceInt raised;   // per instantiation
  const hipError_t attr = ensure_dynamic_lds(raised, (const void*)kern, LDS);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(kern, dim3((unsigned)nblocks), dim3(THREADS), LDS, stream, g, tiles_m, tiles_n);
  return hipGetLastError();
}

// Large un-gathered bf16 problems take 256x256 block tiles (half the LDS and L2 traffic per flop);
// everything else takes 128x128 tiles, which also fill the chip at small sizes.
inline bool use_big_tiles(const GemmArgs& g) {
  const long tiles = (long)((g.M + 255) / 256) * ((g.N + 255) / 256) * g.batch;
  return !g.gatherA && !g.gatherB && g.N >= 256 && tiles >= 512;
}

// every row of both bf16 operands starts on a 16-byte boundary (the direct-to-LDS loads move 16 bytes per lane)
inline bool aligned16(const GemmArgs& g) {
  return g.lda % 8 == 0 && g.ldb % 8 == 0 && (((uintptr_t)g.A | (uintptr_t)g.B) & 15) == 0 && g.strideA % 8 == 0 && g.strideB % 8 == 0 &&
         g.strideA2 % 8 == 0 && g.strideB2 % 8 == 0;
}

template <typename In, int EPI>
hipError_t launch_t(const GemmArgs& g, hipStream_t stream) {
  if constexpr (std::is_same<In, bf16_t>::value && EPI == EPI_STORE_F64) {
    // fp64 results from bf16 rows (gathered or not): the direct-to-LDS kernel when the shape allows it
    if (aligned16(g) && g.K % 32 == 0 && g.K >= 32 && g.M >= 1 && g.N >= 1 && (long)g.M * g.N * g.batch >= 128L * 128 * 64)
      return launch_gram_dma(g, stream);
  }
  if (g.gatherA || g.gatherB) return launch_cfg<In, EPI, true, 2>(g, stream);
  if constexpr (std::is_same<In, bf16_t>::value && EPI != EPI_STORE_F64) {
    if (use_big_tiles(g)) {
      // byte offsets inside an image (rows padded to whole tiles included) have to fit 31 bits
      if (g.K % 64 == 0 && g.K >= 128 && g.M >= 1 && g.N >= 1 && ((long)(g.M + 256) * g.lda + g.K) * 2 < 0x7fffffffL &&
          ((long)(g.N + 256) * g.ldb + g.K) * 2 < 0x7fffffffL && aligned16(g))
        return launch_ring<EPI>(g, stream);
      return launch_cfg<In, EPI, false, 4>(g, stream);
    }
  }
  return launch_cfg<In, EPI, false, 2>(g, stream);
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

int gemm_tiles_n(int N) { return (N + 127) / 128; }


hipError_t launch_gemm_nt(const GemmArgs& g, int dtype, hipStream_t stream) {
  return dtype == DT_BF16 ? launch_e<bf16_t>(g, stream) : launch_e<float>(g, stream);
}

}  // namespace covspec
