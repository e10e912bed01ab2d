// Draft-side vocabulary pass (paper Sec. III-B, margin and gating equations; Sec. III-C, fan-out equation and
// the bonus-token candidate rule): for every drafted position one read of the draft logits yields the softmax
// statistics, the two largest probabilities (margin, gate) and the F_j words with the largest logits other
// than the drafted token.
//
// Scan kernel, one workgroup per chunk of 8192 words of one row: every thread keeps its 32 logits in
// registers, accumulates the streaming softmax statistics, and the chunk's K = F_0 + 1 largest logits are
// found by a threshold instead of K rounds of a block-wide argmax: tau = the K-th largest of the 64 quad
// maxima, so at least K logits are >= tau and, for continuous data, only about K more; those few go to a list
// in LDS that one wave ranks by all-pairs comparison.  A list that overflows (many equal logits, or fewer than
// K quads with data) falls back to K rounds of block-wide argmax over the registers: slower, same result.
// Merge kernel, one wave per row: combines the chunks' statistics in fp64, merges their candidate lists,
// evaluates the margin and writes gate and candidates.
#include "common.h"
#include "kernels.h"
#include "vocab.h"

namespace covspec {

namespace {

typedef unsigned long long u64;

constexpr int DTH = 256;                  // threads of the scan kernel
constexpr int EPT = 32;                   // logits per thread
constexpr int DCL = DTH * EPT;            // words per chunk
constexpr int KMAX = 33;                  // F_0 <= 32, plus one for the drafted token
constexpr int LISTCAP = 64;               // threshold list: one entry per lane of the ranking wave
constexpr int MAXCHUNKS = 64;             // the merge kernel keeps chunks * K keys in LDS

// (order key of the logit, ~word): larger logit first, lower word first among equal logits; never 0 for a real entry
__device__ __forceinline__ u64 pack_key(float v, int w) { return ((u64)float_order_key(v) << 32) | (u64)(0xFFFFFFFFu - (uint32_t)w); }
__device__ __forceinline__ int key_word(u64 k) { return (int)(0xFFFFFFFFu - (uint32_t)(k & 0xFFFFFFFFull)); }
__device__ __forceinline__ float key_value(u64 k) {
  const uint32_t o = (uint32_t)(k >> 32);
  return __uint_as_float((o & 0x80000000u) ? (o ^ 0x80000000u) : ~o);
}

// lane's rank among the n <= 64 distinct keys of an LDS array: the number of keys greater than its own
__device__ __forceinline__ int wave_rank(const u64* keys, int n, u64 mine) {
  int rank = 0;
  int j = 0;
  for (; j + 8 <= n; j += 8) {        // eight broadcast reads in flight
    u64 k[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) k[q] = keys[j + q];
#pragma unroll
    for (int q = 0; q < 8; ++q) rank += k[q] > mine ? 1 : 0;
  }
  for (; j < n; ++j) rank += keys[j] > mine ? 1 : 0;
  return rank;
}

struct FanTable { unsigned char f[64]; };   // F_j by position inside the drafted segment

// stats[(row * chunks + c) * 2 + {0,1}] = reference, sum (base-2 domain); top[(row * chunks + c) * KMAX + r],
// r < K: the chunk's r-th largest logit as a packed key, 0 where the chunk has fewer.
template <int DT>
__global__ __launch_bounds__(DTH) void draft_scan_kernel(const void* __restrict__ zd, int V, int chunks, int K,
                                                         double* __restrict__ stats, u64* __restrict__ top) {
  constexpr int N = LogitVec<DT>::N;
  constexpr int NV = EPT / N;
  __shared__ u64 gkey[64];
  __shared__ u64 list[LISTCAP];
  __shared__ u64 wbest[DTH / 64];
  __shared__ double red[DTH / 64][2];
  __shared__ float sh_tau;
  __shared__ int sh_cnt;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const long row = blockIdx.y;
  const int c = blockIdx.x;
  const int w0 = c * DCL, w1 = min(V, w0 + DCL);      // V % N == 0: whole vectors only
  const long base = row * (long)V;

  // a slot without a word, or with a NaN logit, compares false against every threshold and is skipped by max
  float v[EPT];
  uint32_t valid = 0u;                 // whole vectors: bits i*N .. i*N+N-1
  float cref = -INFINITY, sum = 0.f, tmax = -INFINITY;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int w = w0 + (i * DTH + tid) * N;
    if (w < w1) {
      float t[N];
      LogitVec<DT>::load(zd, base + w, t);
      tmax = fmaxf(tmax, online_add<N>(cref, sum, t));
      valid |= ((N == 8 ? 0xFFu : 0xFu) << (i * N));
#pragma unroll
      for (int e = 0; e < N; ++e) v[i * N + e] = t[e];
    } else {
#pragma unroll
      for (int e = 0; e < N; ++e) v[i * N + e] = __builtin_nanf("");
    }
  }
  auto word_of = [&](int e) { return w0 + ((e / N) * DTH + tid) * N + (e % N); };

  // quad maxima -> tau
  tmax = fmaxf(tmax, __shfl_xor(tmax, 1, 64));
  tmax = fmaxf(tmax, __shfl_xor(tmax, 2, 64));
  if ((lane & 3) == 0) gkey[tid >> 2] = ((u64)float_order_key(tmax) << 32) | (u64)(63 - (tid >> 2));
  if (tid == 0) sh_cnt = 0;
  {
    double mm, ss;
    block_combine<DTH / 64>(cref, sum, red, mm, ss);      // its barrier also publishes gkey and sh_cnt
    if (tid == 0) { stats[(row * chunks + c) * 2] = mm; stats[(row * chunks + c) * 2 + 1] = ss; }
  }
  // the two single-wave steps rotate over the waves with the chunk, so that no one SIMD of the compute unit
  // carries them for every resident workgroup
  const int rw = (int)((blockIdx.x + blockIdx.y) & 3u);
  if (wv == rw) {
    const u64 mine = gkey[lane];
    if (wave_rank(gkey, 64, mine) == K - 1) sh_tau = key_value(mine);     // ranks are a permutation of 0..63; K <= 64
  }
  __syncthreads();
  const float tau = sh_tau;
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    if (v[e] >= tau) {
      const int pos = atomicAdd(&sh_cnt, 1);
      if (pos < LISTCAP) list[pos] = pack_key(v[e], word_of(e));
    }
  }
  __syncthreads();
  const int n = sh_cnt;
  u64* out = top + (row * chunks + c) * KMAX;
  if (n <= LISTCAP) {
    if (wv == ((rw + 2) & 3)) {
      const u64 mine = lane < n ? list[lane] : 0ull;
      const int rank = wave_rank(list, n, mine);
      if (lane < n && rank < K) out[rank] = mine;
      if (lane >= n && lane < K) out[lane] = 0ull;        // fewer than K logits in the chunk
    }
    return;
  }
  // fallback: K rounds of block-wide argmax over the registers
  uint32_t alive = valid;
  for (int r = 0; r < K; ++r) {
    u64 best = 0ull;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      if (((alive >> e) & 1u) && v[e] == v[e]) {
        const u64 k = pack_key(v[e], word_of(e));
        best = k > best ? k : best;
      }
    }
    best = wave_max(best);
    if (lane == 0) wbest[wv] = best;
    __syncthreads();
    u64 b = wbest[0];
#pragma unroll
    for (int k = 1; k < DTH / 64; ++k) b = wbest[k] > b ? wbest[k] : b;
    if (b != 0ull) {
      const int rel = key_word(b) - w0;                   // in [0, DCL)
      const int vec = rel / N;
      if ((vec % DTH) == tid) alive &= ~(1u << ((vec / DTH) * N + rel % N));
    }
    if (tid == 0) out[r] = b;
    __syncthreads();
  }
}

// One wave per row.
__global__ __launch_bounds__(64) void draft_merge_kernel(const double* __restrict__ stats, const u64* __restrict__ top,
                                                         const int32_t* __restrict__ tok, int L, int V, int chunks, int K, int F0,
                                                         FanTable fan, float gamma, float* __restrict__ margin_out,
                                                         int32_t* __restrict__ gate_out, int32_t* __restrict__ cand_out) {
  extern __shared__ u64 pool[];                 // chunks * K keys
  __shared__ u64 sorted[KMAX];
  const int row = blockIdx.x, lane = threadIdx.x;
  const int total = chunks * K;
  for (int i = lane; i < total; i += 64) pool[i] = top[((long)row * chunks + i / K) * KMAX + i % K];
  double m = 0.0, s = 0.0;
  for (int c = lane; c < chunks; c += 64) {
    const double m2 = stats[((long)row * chunks + c) * 2], s2 = stats[((long)row * chunks + c) * 2 + 1];
    if (s2 > 0.0) {
      if (s > 0.0) combine_pair(m, s, m2, s2);
      else { m = m2; s = s2; }
    }
  }
  wave_combine(m, s);
  __syncthreads();
  for (int r = 0; r < K; ++r) {
    u64 best = 0ull;
    int bi = -1;
    for (int i = lane; i < total; i += 64) {
      const u64 k = pool[i];
      if (k > best) { best = k; bi = i; }
    }
    const u64 wb = wave_max(best);
    if (wb != 0ull && best == wb) pool[bi] = 0ull;     // keys are distinct: exactly one lane
    if (lane == 0) sorted[r] = wb;
    __syncthreads();
  }
  if (lane == 0) {
    // margin = p_(1) - p_(2); V >= 2, so both exist
    const double y1 = (double)key_value(sorted[0]) * (double)kLog2e, y2 = (double)key_value(sorted[1]) * (double)kLog2e;
    const float mf = (float)((exp2(y1 - m) - exp2(y2 - m)) / s);
    margin_out[row] = mf;
    gate_out[row] = mf >= gamma ? 0 : 1;
  }
  if (F0 > 0) {
    const int y = tok[row];
    const u64 mine = lane < K ? sorted[lane] : 0ull;
    const u64 hit = __ballot(mine != 0ull && key_word(mine) == y);
    const int pos_y = hit ? __ffsll((long long)hit) - 1 : K;
    const int Fj = fan.f[row % L];
    if (lane < F0) {
      const int j = lane + (lane >= pos_y ? 1 : 0);    // <= F0 = K - 1
      const u64 k = sorted[j];
      cand_out[(long)row * F0 + lane] = (lane < Fj && k != 0ull) ? key_word(k) : -1;
    }
  }
}

}  // namespace

int draft_chunks(int V) { return (V + DCL - 1) / DCL; }
int draft_max_vocab() { return MAXCHUNKS * DCL; }

size_t draft_workspace_bytes(int S, int L, int V) {
  const size_t rows = (size_t)S * L, chunks = (size_t)draft_chunks(V);
  return rows * chunks * 2 * sizeof(double) + rows * chunks * KMAX * sizeof(u64) + 512;
}

hipError_t launch_draft(const void* zd, const int32_t* tok, int S, int L, int V, int dtype, int F0, const int* fanout, float gamma,
                        float* margin, int32_t* gate, int32_t* cand, void* ws, hipStream_t st) {
  const int chunks = draft_chunks(V);
  const long rows = (long)S * L;
  if (S < 1 || L < 1 || L > 64 || V < 2 || rows > 65535 || chunks > MAXCHUNKS || F0 < 0 || F0 > KMAX - 1) return hipErrorInvalidValue;
  const int K = F0 + 1 < 2 ? 2 : F0 + 1;
  FanTable fan;
  for (int j = 0; j < 64; ++j) fan.f[j] = (unsigned char)(j < L ? fanout[j] : 0);
  double* stats = (double*)ws;
  u64* top = (u64*)(stats + (size_t)rows * chunks * 2);
  if (dtype == DT_BF16)
    hipLaunchKernelGGL((draft_scan_kernel<DT_BF16>), dim3(chunks, (unsigned)rows), dim3(DTH), 0, st, zd, V, chunks, K, stats, top);
  else if (dtype == DT_F16)
    hipLaunchKernelGGL((draft_scan_kernel<DT_F16>), dim3(chunks, (unsigned)rows), dim3(DTH), 0, st, zd, V, chunks, K, stats, top);
  else
    hipLaunchKernelGGL((draft_scan_kernel<DT_F32>), dim3(chunks, (unsigned)rows), dim3(DTH), 0, st, zd, V, chunks, K, stats, top);
  hipLaunchKernelGGL(draft_merge_kernel, dim3((unsigned)rows), dim3(64), (size_t)chunks * K * sizeof(u64), st, (const double*)stats,
                     (const u64*)top, tok, L, V, chunks, K, F0, fan, gamma, margin, gate, cand);
  return hipGetLastError();
}

}  // namespace covspec
