// Speculative verification over the vocabulary (paper Sec. II-A: softmax of the draft and target logits,
// acceptance probability of each drafted token, residual distribution after the first rejection).
//
// Per sequence s and drafted position tau the two logit rows z_t, z_d [V] are read ONCE by the statistics
// pass (reference and sum of exponentials of both, fp32 exponentials, partial results per chunk so that a
// few rows still fill the device); the acceptance pass combines them in fp64, evaluates
// alpha = min(1, p_t(y)/p_d(y)) at the drafted token, finds the first rejection and notes that row's
// statistics; only that one row per sequence is read again, in fp64: once for the exact sums and the chunk
// masses of max(p_t - p_d, 0), then, inside the one chunk that holds u_res * (total residual mass), for the
// inverse-CDF search of the correction.  Everything is HBM-bound streaming except the fp64 exponentials of the
// residual pass (2 per word, one row per sequence).
#include "common.h"
#include "kernels.h"
#include "vocab.h"

namespace covspec {

namespace {

constexpr int VT = 256;            // threads of the streaming kernels

// stats[(row * chunks + c) * 4 + {0,1,2,3}] = ref_t, sum_t, ref_d, sum_d (base-2 domain) over words [c*clen, min(V, (c+1)*clen))
template <int DT>
__global__ __launch_bounds__(VT) void verify_stats_kernel(const void* __restrict__ zt, const void* __restrict__ zd, int V, int clen,
                                                          int chunks, double* __restrict__ stats) {
  constexpr int N = LogitVec<DT>::N;
  __shared__ double red[2][VT / 64][2];
  const long row = blockIdx.y;
  const int c = blockIdx.x;
  const int w0 = c * clen, w1 = min(V, w0 + clen);
  const long base = row * (long)V;
  float mt = -INFINITY, st = 0.f, md = -INFINITY, sd = 0.f;
  // V, clen % N == 0: whole vectors only.  (Two vectors per trip with all loads issued first, and twice the
  // workgroups, both measured slower: the pass runs at the rate the memory system gives one resident round.)
  for (int w = w0 + threadIdx.x * N; w < w1; w += VT * N) {
    float a[N], b[N];
    LogitVec<DT>::load(zt, base + w, a);
    LogitVec<DT>::load(zd, base + w, b);
    online_add<N>(mt, st, a);
    online_add<N>(md, sd, b);
  }
  double mm, ss;
  block_combine<VT / 64>(mt, st, red[0], mm, ss);
  if (threadIdx.x == 0) { stats[(row * chunks + c) * 4] = mm; stats[(row * chunks + c) * 4 + 1] = ss; }
  block_combine<VT / 64>(md, sd, red[1], mm, ss);
  if (threadIdx.x == 0) { stats[(row * chunks + c) * 4 + 2] = mm; stats[(row * chunks + c) * 4 + 3] = ss; }
}

// One wave per sequence, one lane per drafted position: row statistics from the chunk partials, alpha at the
// drafted token, first rejection.  rowmax[s * 4 + {0,1}] = the rejected row's references brought back to the
// natural domain, i.e. its maximum logits to within rounding: the shift the fp64 passes below use (any value
// near the maximum serves, as long as every pass uses the same), [2] = the ratio of the two streaming sums;
// untouched when nothing is rejected.
template <int DT>
__global__ __launch_bounds__(64) void verify_accept_kernel(const void* __restrict__ zt, const void* __restrict__ zd,
                                                           const int32_t* __restrict__ tok, const float* __restrict__ u_acc, int L,
                                                           int V, int chunks, const double* __restrict__ stats,
                                                           int32_t* __restrict__ n_acc, float* __restrict__ alpha_out,
                                                           double* __restrict__ rowmax) {
  const int s = blockIdx.x, lane = threadIdx.x;
  int first = L;
  for (int t0 = 0; t0 < L; t0 += 64) {
    const int t = t0 + lane;
    bool rejected = false;
    double m[2] = {0.0, 0.0}, sum[2] = {0.0, 0.0};
    if (t < L) {
      const long row = (long)s * L + t;
      for (int q = 0; q < 2; ++q)
        for (int c = 0; c < chunks; ++c) {
          const double m2 = stats[(row * chunks + c) * 4 + 2 * q], s2 = stats[(row * chunks + c) * 4 + 2 * q + 1];
          if (s2 > 0.0) {
            if (sum[q] > 0.0) combine_pair(m[q], sum[q], m2, s2);
            else { m[q] = m2; sum[q] = s2; }
          }
        }
      int y = tok[row];
      y = y < 0 ? 0 : (y >= V ? V - 1 : y);     // never index outside the row
      const double pt = exp2(LogitVec<DT>::at(zt, row * V + y) * (double)kLog2e - m[0]) / sum[0];
      const double pd = exp2(LogitVec<DT>::at(zd, row * V + y) * (double)kLog2e - m[1]) / sum[1];
      const double a = pd > 0.0 ? fmin(1.0, pt / pd) : 1.0;
      const float af = (float)a;
      if (alpha_out) alpha_out[row] = af;
      rejected = !(u_acc[row] < af);
    }
    const unsigned long long mask = __ballot(rejected);
    if (mask != 0ull) {
      const int fl = __ffsll((long long)mask) - 1;
      first = t0 + fl;
      if (lane == fl) {
        rowmax[s * 4] = m[0] / (double)kLog2e;
        rowmax[s * 4 + 1] = m[1] / (double)kLog2e;
        // estimate of (sum_w exp(z_t - shift_t)) / (sum_w exp(z_d - shift_d)), good to the ~1e-6 of the streaming sums
        rowmax[s * 4 + 2] = sum[0] / sum[1];
      }
      break;      // uniform: the ballot is the same in every lane
    }
  }
  if (lane == 0) n_acc[s] = first;
}

// The one fp64 pass over the rejected row of each sequence, per chunk: exact sums S_t, S_d of the exponentials
// (the residual is a difference of the two distributions, and the fp32 sums of the first pass, good to ~1e-6,
// would move its cumulative sums by more than a flat residual's single words) and, in the same pass, the
// chunk's residual mass.  max(p_t - p_d, 0) = max(e_t - kappa e_d, 0) / S_t with kappa = S_t / S_d, which is not
// known before the pass ends; but the mass is A - kappa B with A, B the sums of e_t, e_d over the words where
// e_t > kappa e_d, and an error delta in the kappa that picks those words changes the mass only to second
// order (a word that changes sides carries a residual below delta e_d).  So the words are picked with the
// streaming estimate (delta ~ 1e-6, mass error ~ 1e-12 relative) and A, B are combined with the exact kappa
// afterwards.  rowsum[(s * rchunks + c) * 4 + {0,1,2,3}] = S_t, S_d, A, B of the chunk.
template <int DT>
__global__ __launch_bounds__(VT) void verify_rowpass64_kernel(const void* __restrict__ zt, const void* __restrict__ zd, int L, int V,
                                                              int rlen, int rchunks, const int32_t* __restrict__ n_acc,
                                                              const double* __restrict__ rowmax, double* __restrict__ rowsum) {
  __shared__ double red[4][VT / 64];
  const int s = blockIdx.y, c = blockIdx.x;
  const int t = n_acc[s];
  if (t >= L) return;
  const long base = ((long)s * L + t) * V;
  const int w0 = c * rlen, w1 = min(V, w0 + rlen);
  const double mt = rowmax[s * 4], md = rowmax[s * 4 + 1], kap = rowmax[s * 4 + 2];
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
  for (int w = w0 + threadIdx.x; w < w1; w += VT) {
    const double et = exp(LogitVec<DT>::at(zt, base + w) - mt);
    const double ed = exp(LogitVec<DT>::at(zd, base + w) - md);
    acc[0] += et;
    acc[1] += ed;
    if (et > kap * ed) { acc[2] += et; acc[3] += ed; }     // equal rows: kap == 1 and et == ed exactly, nothing is picked
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) acc[q] = wave_sum(acc[q]);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  if (lane == 0) {
#pragma unroll
    for (int q = 0; q < 4; ++q) red[q][wv] = acc[q];
  }
  __syncthreads();
  if (threadIdx.x < 4) {
    const int q = threadIdx.x;
    double tot = 0.0;
    for (int k = 0; k < VT / 64; ++k) tot += red[q][k];
    rowsum[((long)s * rchunks + c) * 4 + q] = tot;
  }
}

// wave 0 of a workgroup (all 64 lanes): the row's (max_t, 1/sum_t, max_d, 1/sum_d) from the chunk sums, into
// LDS.  rchunks <= 64: lane c holds chunk c, butterfly sums (the same order wherever this is called).  Returns
// the residual mass of chunk `lane`, A / S_t - B / S_d (0 for lanes beyond the chunks).
__device__ __forceinline__ double combine_rowstat(const double* __restrict__ rowmax, const double* __restrict__ rowsum, int s, int rchunks,
                                                  double* sh4) {
  const int lane = threadIdx.x & 63;
  const double* rs = rowsum + ((long)s * rchunks + lane) * 4;
  const double st_c = lane < rchunks ? rs[0] : 0.0, sd_c = lane < rchunks ? rs[1] : 0.0;
  const double a_c = lane < rchunks ? rs[2] : 0.0, b_c = lane < rchunks ? rs[3] : 0.0;
  const double st = wave_sum(st_c), sd = wave_sum(sd_c);
  const double ist = 1.0 / st, isd = 1.0 / sd;
  if (lane == 0) { sh4[0] = rowmax[s * 4]; sh4[1] = ist; sh4[2] = rowmax[s * 4 + 1]; sh4[3] = isd; }
  double mass;
  {
#pragma clang fp contract(off)
    const double x = a_c * ist, y = b_c * isd;
    mass = x - y;
  }
  return mass > 0.0 ? mass : 0.0;
}

template <int DT>
__device__ __forceinline__ double residual_at(const void* zt, const void* zd, long i, double mt, double ist, double md, double isd) {
  // each product rounded on its own: contracted into a fused multiply-add the difference of two EQUAL
  // probabilities would come out as rounding noise instead of zero
#pragma clang fp contract(off)
  const double a = exp(LogitVec<DT>::at(zt, i) - mt) * ist;
  const double b = exp(LogitVec<DT>::at(zd, i) - md) * isd;
  const double d = a - b;
  return d > 0.0 ? d : 0.0;
}

// One 1024-thread workgroup per sequence: inverse CDF of the residual in vocabulary order.
template <int DT>
__global__ __launch_bounds__(1024) void verify_sample_kernel(const void* __restrict__ zt, const void* __restrict__ zd, int L, int V,
                                                             int clen, int chunks, const int32_t* __restrict__ n_acc,
                                                             const double* __restrict__ rowmax, const double* __restrict__ rowsum,
                                                             const float* __restrict__ u_res, int32_t* __restrict__ corr) {
  __shared__ double wsum[16];
  __shared__ double sh_prefix, sh_target;
  __shared__ int sh_chunk, sh_found, sh_last;
  __shared__ unsigned long long sh_best;
  const int s = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int t = n_acc[s];
  if (t >= L) { if (tid == 0) corr[s] = -1; return; }
  const long base = ((long)s * L + t) * V;
  __shared__ double sh4[4];
  double pc = 0.0;
  if (tid < 64) pc = combine_rowstat(rowmax, rowsum, s, chunks, sh4);     // this lane's chunk mass (wave 0)
  __syncthreads();
  const double mt = sh4[0], ist = sh4[1], md = sh4[2], isd = sh4[3];
  if (tid < 64) {
    // lane c holds chunk c's residual mass; inclusive scan in lane order, total in lane 63
    double inc = pc;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const double v = __shfl_up(inc, o, 64);
      if (lane >= o) inc += v;
    }
    const double R = __shfl(inc, 63, 64);
    const double target = (double)u_res[s] * R;
    // the first chunk whose cumulative mass passes the target; if rounding leaves the target at the total,
    // the last chunk with any mass
    const unsigned long long over = __ballot(pc > 0.0 && inc > target);
    const unsigned long long mass = __ballot(pc > 0.0);
    int cs = -1;
    if (R > 0.0) cs = over ? __ffsll((long long)over) - 1 : 63 - __clzll((long long)mass);
    if (lane == (cs < 0 ? 0 : cs)) {
      sh_chunk = cs; sh_prefix = inc - pc; sh_target = target; sh_found = 0x7fffffff; sh_last = -1; sh_best = 0ull;
    }
  }
  __syncthreads();
  const int cs = sh_chunk;
  if (cs < 0) {
    // no residual mass (p_t == p_d): argmax p_t, lowest index on ties
    unsigned long long best = 0ull;
    for (int w = tid; w < V; w += 1024) {
      const float z = (float)LogitVec<DT>::at(zt, base + w);   // logits are stored in at most fp32: exact
      const unsigned long long key = ((unsigned long long)float_order_key(z) << 32) | (0xFFFFFFFFu - (uint32_t)w);
      best = key > best ? key : best;
    }
    best = wave_max(best);
    if (lane == 0) atomicMax(&sh_best, best);
    __syncthreads();
    if (tid == 0) corr[s] = (int)(0xFFFFFFFFu - (uint32_t)(sh_best & 0xFFFFFFFFull));
    return;
  }
  // inside the chunk: thread `tid` owns the contiguous words [w0 + tid*per, w0 + (tid+1)*per)
  const int w0 = cs * clen, w1 = min(V, w0 + clen);
  const int per = (w1 - w0 + 1023) / 1024;
  const int a0 = w0 + tid * per, a1 = min(w1, a0 + per);
  double mine = 0.0;
  for (int w = a0; w < a1; ++w) mine += residual_at<DT>(zt, zd, base + w, mt, ist, md, isd);
  // exclusive prefix over the threads (fp64): wave scan, then the 16 wave totals
  double inc = mine;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const double v = __shfl_up(inc, o, 64);
    if (lane >= o) inc += v;
  }
  if (lane == 63) wsum[wv] = inc;
  __syncthreads();
  double before = sh_prefix;
  for (int k = 0; k < wv; ++k) before += wsum[k];
  before += inc - mine;
  // second pass over the own words: the first word at which the running sum passes the target, and the last
  // word with any mass.  A thread that starts beyond the target reports its first word; the minimum over all
  // threads is the crossing.  If rounding leaves the target just past the chunk, the last word with mass is it.
  const double target = sh_target;
  double run = before;
  int hit = 0x7fffffff, last = -1;
  for (int w = a0; w < a1; ++w) {
    const double r = residual_at<DT>(zt, zd, base + w, mt, ist, md, isd);
    if (r > 0.0) last = w;
    run += r;
    if (hit == 0x7fffffff && run > target && r > 0.0) hit = w;
  }
  if (hit != 0x7fffffff) atomicMin(&sh_found, hit);
  if (last >= 0) atomicMax(&sh_last, last);
  __syncthreads();
  if (tid == 0) corr[s] = sh_found != 0x7fffffff ? sh_found : (sh_last >= 0 ? sh_last : w1 - 1);
}

}  // namespace

void verify_plan(int S, int L, int V, int dtype, int* clen, int* chunks) {
  // chunks per row so that even a few rows give the streaming kernel ~1024 workgroups; chunk length a
  // multiple of what one pass of the workgroup covers
  const int vec = dtype == DT_F32 ? 4 : 8;
  const int step = VT * vec;
  long rows = (long)S * L;
  int want = (int)((1024 + rows - 1) / rows);
  if (want < 1) want = 1;
  if (want > 64) want = 64;
  int len = (V + want - 1) / want;
  len = (len + step - 1) / step * step;
  *clen = len;
  *chunks = (V + len - 1) / len;
}

// the fp64 passes read one row per sequence: their own, finer split (~2048 workgroups, at most 64 chunks a row)
static void residual_plan(int S, int V, int* rlen, int* rchunks) {
  int want = (2048 + S - 1) / S;
  if (want < 1) want = 1;
  if (want > 64) want = 64;
  int len = (V + want - 1) / want;
  len = (len + VT - 1) / VT * VT;
  *rlen = len;
  *rchunks = (V + len - 1) / len;
}

size_t verify_workspace_bytes(int S, int L, int V, int dtype) {
  int clen, chunks, rlen, rchunks;
  verify_plan(S, L, V, dtype, &clen, &chunks);
  residual_plan(S, V, &rlen, &rchunks);
  return ((size_t)S * L * chunks * 4 + (size_t)S * 4 + (size_t)S * rchunks * 4) * sizeof(double) + 512;
}

template <int DT>
static hipError_t launch_verify_t(const void* zt, const void* zd, const int32_t* tok, const float* u_acc, const float* u_res, int S,
                                  int L, int V, int32_t* n_acc, int32_t* corr, float* alpha, void* ws, hipStream_t st) {
  int clen, chunks, rlen, rchunks;
  verify_plan(S, L, V, DT, &clen, &chunks);
  residual_plan(S, V, &rlen, &rchunks);
  double* stats = (double*)ws;                               // [S*L][chunks][4]
  double* rowmax = stats + (size_t)S * L * chunks * 4;       // [S][4]
  double* rowsum = rowmax + (size_t)S * 4;                   // [S][rchunks][4]
  hipLaunchKernelGGL((verify_stats_kernel<DT>), dim3(chunks, S * L), dim3(VT), 0, st, zt, zd, V, clen, chunks, stats);
  hipLaunchKernelGGL((verify_accept_kernel<DT>), dim3(S), dim3(64), 0, st, zt, zd, tok, u_acc, L, V, chunks, (const double*)stats, n_acc,
                     alpha, rowmax);
  hipLaunchKernelGGL((verify_rowpass64_kernel<DT>), dim3(rchunks, S), dim3(VT), 0, st, zt, zd, L, V, rlen, rchunks, (const int32_t*)n_acc,
                     (const double*)rowmax, rowsum);
  hipLaunchKernelGGL((verify_sample_kernel<DT>), dim3(S), dim3(1024), 0, st, zt, zd, L, V, rlen, rchunks, (const int32_t*)n_acc,
                     (const double*)rowmax, (const double*)rowsum, u_res, corr);
  return hipGetLastError();
}

hipError_t launch_verify(const void* zt, const void* zd, const int32_t* tok, const float* u_acc, const float* u_res, int S, int L,
                         int V, int dtype, int32_t* n_acc, int32_t* corr, float* alpha, void* ws, hipStream_t st) {
  if (S < 1 || L < 1 || V < 2 || (long)S * L > 65535) return hipErrorInvalidValue;
  if (dtype == DT_BF16) return launch_verify_t<DT_BF16>(zt, zd, tok, u_acc, u_res, S, L, V, n_acc, corr, alpha, ws, st);
  if (dtype == DT_F16) return launch_verify_t<DT_F16>(zt, zd, tok, u_acc, u_res, S, L, V, n_acc, corr, alpha, ws, st);
  return launch_verify_t<DT_F32>(zt, zd, tok, u_acc, u_res, S, L, V, n_acc, corr, alpha, ws, st);
}

}  // namespace covspec
