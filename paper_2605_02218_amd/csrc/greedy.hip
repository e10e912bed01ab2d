// Greedy residual-update selection (a variant that is not in the paper; it replaces
// the rank-r SVD energy ranking of Sec. III-A.3 by k greedy picks).
//
// Pivoted Cholesky of the token Gram matrix G = Z Z^T in fp64: the residual squared
// norm of token i after projecting out the picked tokens is rho_i; each step picks
// argmax rho (decided on the fp32-rounded value, ties -> lower index), forms the new
// Cholesky column l = (G[:,p] - L L[p,:]^T) / sqrt(rho_p) and updates rho -= l^2.
//
// Three kernels, chosen by launch_greedy from the values each would move: the right-looking panel kernel
// (greedy_panel_kernel, the usual choice), and two left-looking ones for the case that the picks are a small
// part of the rows, on several workgroups per image (greedy_kernel) or one (greedy_single_kernel).
//
// Left-looking on several workgroups (greedy_kernel).  The k steps are dependent, but inside a step the rows are
// independent, so an image is spread over nP/64 workgroups of 64 rows each: a workgroup keeps rho of its rows in
// registers, posts its best (key, rho) per step, all workgroups of the image meet at a
// barrier in global memory (one per step), read the posts, agree on the pivot p, fetch
// the pivot's Cholesky row L[p, 0..t) and extend their own 64 rows of L.  L is stored
// transposed (Lt[t][i]) so that a workgroup's part of a column is one 512-byte run.
// Inside a workgroup lanes are rows and the four waves split the dot product over t.
// Workgroups take (image, slot) from a ticket counter, so the resident ones always form
// whole images plus one partial image that is next in the dispatch order.
#include "common.h"
#include "host_cache.h"
#include "kernels.h"

namespace covspec {

namespace {

constexpr int TPB = 1024;   // finish kernel
constexpr int GR = 64;      // rows per workgroup
constexpr int GT = 256;     // threads per workgroup

struct GreedyCtl {
  ImageBarrier bar;
  unsigned int ticket;   // ctl[0] only
  unsigned int pad;
};

__global__ void greedy_init_kernel(GreedyCtl* ctl, int B) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b < B) { ctl[b].bar.arrived = 0u; ctl[b].bar.failed = 0; ctl[b].ticket = 0u; ctl[b].pad = 0u; }
}

// posts: per image [2][W] keys (u64) then [2][W] rho (fp64), double-buffered by step parity
__global__ __launch_bounds__(GT) void greedy_kernel(const double* __restrict__ G, int n, int nP, int k, double* Lt, int32_t* __restrict__ order,
                                                     float* __restrict__ resid, GreedyCtl* ctl, unsigned long long* posts,
                                                     int* img_status, long long limit_ticks) {
  __shared__ double Lp[4096];
  __shared__ double part[4][GR];
  __shared__ unsigned long long sh_key;
  __shared__ double sh_rho;
  __shared__ int s_flag;
  const int W = nP / GR;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  if (tid == 0) s_flag = (int)atomicAdd(&ctl[0].ticket, 1u);
  __syncthreads();
  const int ticket = s_flag;
  __syncthreads();
  const int b = ticket / W, slot = ticket - b * W;
  GreedyCtl* cb = ctl + b;
  const double* Gb = G + (long)b * nP * nP;
  double* Ltb = Lt + (long)b * k * nP;
  unsigned long long* keys = posts + (long)b * 4 * W;       // [2][W]
  double* rhos = (double*)(keys + 2 * W);                   // [2][W]
  const int i = slot * GR + lane;                           // this lane's row (all four waves hold a copy)

  double rho = (i < n) ? Gb[(long)i * nP + i] : 0.0;
  bool picked = !(i < n);
  unsigned int target = 0;
  bool alive = true;

  for (int t = 0; t < k && alive; ++t) {
    // ---- local argmax of float(rho) over the unpicked rows, lowest index on ties (wave 0 suffices)
    if (w == 0) {
      unsigned long long key = 0ull;
      if (!picked) key = ((unsigned long long)float_order_key((float)rho) << 32) | (0xFFFFFFFFu - (uint32_t)i);
      const unsigned long long best = wave_max(key);
      const unsigned long long bal = __ballot(key == best && key != 0ull);
      if (best != 0ull && lane == (int)__ffsll((long long)bal) - 1) {
        keys[(t & 1) * W + slot] = best;
        rhos[(t & 1) * W + slot] = rho;
      }
      if (best == 0ull && lane == 0) keys[(t & 1) * W + slot] = 0ull;
    }
    target += (unsigned int)W;
    alive = image_barrier_wait(&cb->bar, target, &s_flag, limit_ticks);
    if (!alive) break;
    // ---- global argmax over the posts
    if (w == 0) {
      unsigned long long key = 0ull;
      double r = 0.0;
      for (int q = lane; q < W; q += 64) {
        const unsigned long long kq = keys[(t & 1) * W + q];
        if (kq > key) { key = kq; r = rhos[(t & 1) * W + q]; }
      }
      const unsigned long long best = wave_max(key);
      const unsigned long long bal = __ballot(key == best);
      if (lane == (int)__ffsll((long long)bal) - 1) { sh_key = best; sh_rho = r; }
    }
    __syncthreads();
    const int p = (int)(0xFFFFFFFFu - (uint32_t)(sh_key & 0xFFFFFFFFull));
    const double rp = sh_rho;
    if ((unsigned)p >= (unsigned)n) {   // cannot happen with consistent posts; never index with it
      if (tid == 0) __hip_atomic_store(&cb->bar.failed, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      alive = false;
      break;
    }
    if (p == i) picked = true;
    for (int q = tid; q < t; q += GT) Lp[q] = Ltb[(long)q * nP + p];
    __syncthreads();
    // ---- dot products: wave w takes q = w, w+4, ...
    double d0 = 0.0, d1 = 0.0;
    {
      const double* col = Ltb + i;
      int q = w;
      // eight loads in flight per wave: the step lives on their latency
      for (; q + 28 < t; q += 32) {
        double v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = col[(long)(q + 4 * u) * nP];
#pragma unroll
        for (int u = 0; u < 8; u += 2) {
          d0 = fma(v[u], Lp[q + 4 * u], d0);
          d1 = fma(v[u + 1], Lp[q + 4 * u + 4], d1);
        }
      }
      for (; q + 4 < t; q += 8) {
        d0 = fma(col[(long)q * nP], Lp[q], d0);
        d1 = fma(col[(long)(q + 4) * nP], Lp[q + 4], d1);
      }
      if (q < t) d0 = fma(col[(long)q * nP], Lp[q], d0);
    }
    part[w][lane] = d0 + d1;
    __syncthreads();
    const double piv = rp > 0.0 ? rp : 0.0;
    const double root = sqrt(piv);
    const double dot = (part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]);
    const double colv = (piv > 0.0 && i < n) ? (Gb[(long)p * nP + i] - dot) / root : 0.0;
    if (w == 0) Ltb[(long)t * nP + i] = colv;
    rho -= colv * colv;
    if (slot == 0 && tid == 0) { order[(long)b * k + t] = p; resid[(long)b * k + t] = (float)rp; }
  }
  if (!alive && slot == 0) {
    // a wait ran out: leave valid (distinct) positions and poisoned residuals behind
    const float qnan = __uint_as_float(0x7fc00000u);
    for (int t = tid; t < k; t += GT) { order[(long)b * k + t] = t; resid[(long)b * k + t] = qnan; }
    if (img_status && tid == 0) img_status[b] = 1;
  }
}

// One 1024-thread workgroup per image (no barriers between workgroups), left-looking: used when the batch alone
// fills the device and the picks are a small part of the rows (see the right-looking kernel below).
constexpr int RPT = 4;  // rows per thread: n <= 4096

__global__ __launch_bounds__(TPB) void greedy_single_kernel(const double* __restrict__ G, int n, int nP, int k,
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
    // The columns picked so far are re-read from L2 / the memory-side cache at every step; the step lives on the
    // latency of those loads, so sixteen of them are issued before the first is used.
    {
      constexpr int UQ = 16;
      int q = 0;
      for (; q + UQ <= t; q += UQ) {
#pragma unroll
        for (int s = 0; s < RPT; ++s) {
          if (tid + TPB * s < n) {
            double v[UQ];
#pragma unroll
            for (int u = 0; u < UQ; ++u) v[u] = Ltb[(long)(q + u) * nP + tid + TPB * s];
            double d0 = 0.0, d1 = 0.0;
#pragma unroll
            for (int u = 0; u < UQ; u += 2) {
              d0 = fma(v[u], Lp[q + u], d0);
              d1 = fma(v[u + 1], Lp[q + u + 1], d1);
            }
            dot[s] += d0 + d1;
          }
        }
      }
      for (; q < t; ++q) {
        const double lp = Lp[q];
        const double* row = Ltb + (long)q * nP + tid;
#pragma unroll
        for (int s = 0; s < RPT; ++s)
          if (tid + TPB * s < n) dot[s] = fma(row[TPB * s], lp, dot[s]);
      }
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

// Right-looking in blocks of BK picks, an image of up to 4096 rows spread over W workgroups of 1024 threads (thread
// tid owns the NR rows tid, tid + 1024, ...).  The residual matrix R = G - L L^T is kept in global memory IN PLACE of G and
// brought up to date once per block by a rank-BK update on the MFMA; inside a block a new column is the pivot's
// row of R minus the product with the block's earlier columns, which live in LDS.  The left-looking kernels above
// re-read every earlier column at every step (k^2 n / 2 values); this one reads one row of R per step and reads
// and writes R once per block (up to 2 n^2 k / BK values), which is less unless k is a small part of n.
// Every workgroup of the image runs the BK picks of a block redundantly (same loads, same arithmetic, hence the
// same decisions: nothing is exchanged), then the workgroups meet at the image's barrier, each brings its own
// 16-row bands of R up to date, and they meet again before the next block reads rows of R: two barriers per
// block instead of one per pick, and the device's bandwidth on the update instead of one workgroup's.
// Dynamic LDS: BK * nP doubles; workgroups take (image, slot) from the ticket counter.
// Maximum of one 64-bit key per lane over the wave with DPP moves (no LDS round trips): quads, then shifts by 4 and
// 8 inside a row of 16 lanes, then the last lane of a row broadcast into the next row (rows 1 and 3) and lane 31
// into rows 2 and 3, which leaves the maximum in lane 63.  Lanes without a source take 0, the identity for keys.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ unsigned long long dpp_key(unsigned long long v) {
  const unsigned lo = __builtin_amdgcn_update_dpp(0u, (unsigned)v, CTRL, ROW_MASK, 0xf, false);
  const unsigned hi = __builtin_amdgcn_update_dpp(0u, (unsigned)(v >> 32), CTRL, ROW_MASK, 0xf, false);
  return ((unsigned long long)hi << 32) | lo;
}
__device__ __forceinline__ unsigned long long wave_max_key(unsigned long long v) {
  unsigned long long o;
  o = dpp_key<0xb1, 0xf>(v); v = o > v ? o : v;      // quad_perm [1,0,3,2]
  o = dpp_key<0x4e, 0xf>(v); v = o > v ? o : v;      // quad_perm [2,3,0,1]
  o = dpp_key<0x114, 0xf>(v); v = o > v ? o : v;     // row_shr:4
  o = dpp_key<0x118, 0xf>(v); v = o > v ? o : v;     // row_shr:8
  o = dpp_key<0x142, 0xa>(v); v = o > v ? o : v;     // row_bcast:15 into rows 1 and 3
  o = dpp_key<0x143, 0xc>(v); v = o > v ? o : v;     // row_bcast:31 into rows 2 and 3
  const unsigned lo = __builtin_amdgcn_readlane((unsigned)v, 63), hi = __builtin_amdgcn_readlane((unsigned)(v >> 32), 63);
  return ((unsigned long long)hi << 32) | lo;
}

template <int BK, int NR>
__global__ __launch_bounds__(TPB) void greedy_panel_kernel(double* G, int n, int nP, int k, int W, int32_t* __restrict__ order,
                                                            float* __restrict__ resid, GreedyCtl* ctl, int* img_status,
                                                            long long limit_ticks) {
  extern __shared__ double Lblk[];        // [BK][nP]
  __shared__ unsigned long long red[2][16];   // per wave: its best key and that row's residual, double-buffered by
  __shared__ double red_rho[2][16];           // step parity so that a step needs one barrier only
  __shared__ int s_flag;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, i16 = lane & 15, kq = lane >> 4;
  if (tid == 0) s_flag = (int)atomicAdd(&ctl[0].ticket, 1u);
  __syncthreads();
  const int ticket = s_flag;
  __syncthreads();
  const int b = ticket / W, slot = ticket - b * W;
  GreedyCtl* cb = ctl + b;
  double* R = G + (long)b * nP * nP;

  double rho[NR];
  bool picked[NR];
#pragma unroll
  for (int s = 0; s < NR; ++s) {
    const int i = tid + TPB * s;
    rho[s] = (i < n) ? R[(long)i * nP + i] : 0.0;
    picked[s] = !(i < n);
  }
  for (int e = tid; e < BK * nP; e += TPB) Lblk[e] = 0.0;
  unsigned int target = 0;
  bool alive = true;
  // the diagonal is read above and R is first written at the end of block 0, behind a barrier
  __syncthreads();

  for (int t = 0; t < k; ++t) {
    const int jj = t % BK, par = t & 1;
    // ---- argmax over the unpicked rows of float(rho), lowest index on ties.  Keys are distinct, so exactly one
    //      lane of a wave holds the wave's best and posts it with its residual.  One barrier per step: what a
    //      step writes besides is read only behind the next step's barrier, and the posts alternate buffers.
    unsigned long long best = 0ull;
    double brho = 0.0;
#pragma unroll
    for (int s = 0; s < NR; ++s) {
      if (!picked[s]) {
        const unsigned long long key =
            ((unsigned long long)float_order_key((float)rho[s]) << 32) | (0xFFFFFFFFu - (uint32_t)(tid + TPB * s));
        if (key > best) { best = key; brho = rho[s]; }
      }
    }
    {
      const unsigned long long wbest = wave_max_key(best);
      if (wbest == 0ull) { if (lane == 0) red[par][w] = 0ull; }
      else if (best == wbest) { red[par][w] = wbest; red_rho[par][w] = brho; }
    }
    __syncthreads();
    best = red[par][0];
    int wq = 0;
#pragma unroll
    for (int q = 1; q < TPB / 64; ++q)
      if (red[par][q] > best) { best = red[par][q]; wq = q; }
    const double rp = red_rho[par][wq];
    const int p = (int)(0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull));     // < n: k <= n, so an unpicked row exists
    if (best == 0ull || (unsigned)p >= (unsigned)n) {   // never index with anything else
      if (tid == 0) __hip_atomic_store(&cb->bar.failed, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      alive = false;
      break;
    }
    if ((p & (TPB - 1)) == tid) {
#pragma unroll
      for (int s = 0; s < NR; ++s)
        if (s == (p >> 10)) picked[s] = true;
    }
    // ---- the pivot's row of R, minus what this block has already taken out (summed apart, so that the sum
    //      does not wait for the row)
    double c[NR];
#pragma unroll
    for (int s = 0; s < NR; ++s) {
      const int i = tid + TPB * s;
      c[s] = (i < n) ? R[(long)p * nP + i] : 0.0;
    }
    {
      double taken[NR];
#pragma unroll
      for (int s = 0; s < NR; ++s) taken[s] = 0.0;
      for (int q = 0; q < jj; ++q) {
        const double lp = Lblk[q * nP + p];
#pragma unroll
        for (int s = 0; s < NR; ++s) {
          const int i = tid + TPB * s;
          if (i < n) taken[s] = fma(Lblk[q * nP + i], lp, taken[s]);
        }
      }
#pragma unroll
      for (int s = 0; s < NR; ++s) c[s] -= taken[s];
    }
    const double piv = rp > 0.0 ? rp : 0.0;
    const double root = sqrt(piv);
#pragma unroll
    for (int s = 0; s < NR; ++s) {
      const int i = tid + TPB * s;
      const double col = (piv > 0.0 && i < n) ? c[s] / root : 0.0;
      if (i < nP) Lblk[jj * nP + i] = col;
      rho[s] -= col * col;
    }
    if (slot == 0 && tid == 0) { order[(long)b * k + t] = p; resid[(long)b * k + t] = (float)rp; }
    if (jj == BK - 1 && t + 1 < k) {
      // every workgroup of the image has read its last row of the old R (the wait starts with a barrier of
      // the workgroup, behind which the block's columns are complete in LDS)
      target += (unsigned int)W;
      alive = image_barrier_wait(&cb->bar, target, &s_flag, limit_ticks);
      if (!alive) break;
      // ---- R -= Lblk^T Lblk on this workgroup's bands (band ti belongs to slot ti % W); a wave takes four
      //      neighbouring 16 x 16 tiles per trip and requests their 16 values of R before the first MFMA
      const int nt = (n + 15) >> 4;
      const int bands = (nt - slot + W - 1) / W;
      const int ntiles = bands * nt;
      for (int tile0 = 4 * w; tile0 < ntiles; tile0 += 4 * (TPB / 64)) {
        double* out[4];
        double r[4][4];
        int ti[4], tj[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int tile = tile0 + u;
          const int tc = tile < ntiles ? tile : tile0;          // a trailing slot repeats the first tile, result unused
          const int band = tc / nt;
          ti[u] = slot + band * W;
          tj[u] = tc - band * nt;
          // lane (i16, kq), register v: row 16 ti + 4v + kq, column 16 tj + i16 (inside the nP x nP buffer: nP % 64 == 0)
          out[u] = R + (long)(16 * ti[u] + kq) * nP + 16 * tj[u] + i16;
#pragma unroll
          for (int v = 0; v < 4; ++v) r[u][v] = out[u][(long)(4 * v) * nP];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          f64x4_t d = (f64x4_t){0.0, 0.0, 0.0, 0.0};
#pragma unroll
          for (int s4 = 0; s4 < BK / 4; ++s4)
            d = __builtin_amdgcn_mfma_f64_16x16x4f64(Lblk[(4 * s4 + kq) * nP + 16 * ti[u] + i16], Lblk[(4 * s4 + kq) * nP + 16 * tj[u] + i16], d,
                                                     0, 0, 0);
          if (tile0 + u < ntiles) {
#pragma unroll
            for (int v = 0; v < 4; ++v) out[u][(long)(4 * v) * nP] = r[u][v] - d[v];
          }
        }
      }
      // every band is up to date before any workgroup reads a row of R again
      target += (unsigned int)W;
      alive = image_barrier_wait(&cb->bar, target, &s_flag, limit_ticks);
      if (!alive) break;
      for (int e = tid; e < BK * nP; e += TPB) Lblk[e] = 0.0;
      __syncthreads();
    }
  }
  if (!alive && slot == 0) {
    // a wait ran out: leave valid (distinct) positions and poisoned residuals behind
    const float qnan = __uint_as_float(0x7fc00000u);
    for (int t = tid; t < k; t += TPB) { order[(long)b * k + t] = t; resid[(long)b * k + t] = qnan; }
    if (img_status && tid == 0) img_status[b] = 1;
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

size_t greedy_scratch_bytes(int B, int nP) {
  return (size_t)B * sizeof(GreedyCtl) + 256 + (size_t)B * 4 * (nP / GR) * 8;
}

template <int BK, int NR>
static hipError_t launch_panel(double* G, int B, int n, int nP, int k, int W, int32_t* order, float* resid, GreedyCtl* ctl,
                               int* img_status, hipStream_t st) {
  const size_t lds = (size_t)BK * nP * sizeof(double);
  constexpr size_t kLdsMost = 159 * 1024;   // launch_greedy picks BK so that the block's columns stay below this
  if (lds > kLdsMost) return hipErrorInvalidValue;
  static PerDeviceInt raised, cache;   // per instantiation
  hipError_t e = ensure_dynamic_lds(raised, (const void*)greedy_panel_kernel<BK, NR>, kLdsMost);
  if (e != hipSuccess) return e;
  // the workgroups of one image wait for one another, so one image has to fit the device; counted once per device
  // for the largest LDS request, which never overstates what a smaller one gets
  int capacity = 0;
  if ((e = resident_workgroups(cache, greedy_panel_kernel<BK, NR>, TPB, kLdsMost, &capacity)) != hipSuccess) return e;
  if (W > capacity) return hipErrorInvalidValue;
  hipLaunchKernelGGL(greedy_init_kernel, dim3((B + 255) / 256), dim3(256), 0, st, ctl, B);
  hipLaunchKernelGGL((greedy_panel_kernel<BK, NR>), dim3((unsigned)(B * W)), dim3(TPB), lds, st, G, n, nP, k, W, order, resid, ctl,
                     img_status, barrier_limit_ticks());
  return hipGetLastError();
}

hipError_t launch_greedy(double* G, int B, int n, int nP, int k, double* Lt, int32_t* order, float* resid, void* scratch,
                         int* img_status, hipStream_t st) {
  if (nP % GR != 0 || n > nP || n > 4096 || k > n || k > 4096) return hipErrorInvalidValue;
  GreedyCtl* ctl = (GreedyCtl*)scratch;
  // the largest block of picks (a multiple of the MFMA's depth of 4) whose columns fit LDS beside the kernel's few
  // static words
  const size_t lds_cap = 159 * 1024;
  const int BK = (size_t)16 * nP * 8 <= lds_cap ? 16 : (size_t)12 * nP * 8 <= lds_cap ? 12 : (size_t)8 * nP * 8 <= lds_cap ? 8 : 4;
  // values moved: the right-looking kernel reads and writes R once per block that is followed by another, the
  // left-looking ones read every earlier column at every step; the former also has far fewer barriers
  const double right = (double)((k - 1) / BK) * 2.0 * n * n, left = 0.5 * k * k * n;
  if (right <= 2.0 * left) {
    // workgroups per image: measured best with about 128 on the device, at most 32 and (while they fit) at least 4 per image
    const int nt = (n + 15) / 16;
    int Wp = 128 / B;
    if (Wp < 4) Wp = 256 / B < 4 ? 256 / B : 4;
    Wp = Wp < 1 ? 1 : Wp > 32 ? 32 : Wp;
    Wp = Wp > nt ? nt : Wp;
    // rows per thread: at most 1216 rows with blocks of 16, 1664 with 12, 2496 with 8
    if (BK == 16) return n <= TPB ? launch_panel<16, 1>(G, B, n, nP, k, Wp, order, resid, ctl, img_status, st)
                                  : launch_panel<16, 2>(G, B, n, nP, k, Wp, order, resid, ctl, img_status, st);
    if (BK == 12) return launch_panel<12, 2>(G, B, n, nP, k, Wp, order, resid, ctl, img_status, st);
    if (BK == 8) return n <= 2 * TPB ? launch_panel<8, 2>(G, B, n, nP, k, Wp, order, resid, ctl, img_status, st)
                                     : launch_panel<8, 4>(G, B, n, nP, k, Wp, order, resid, ctl, img_status, st);
    return launch_panel<4, 4>(G, B, n, nP, k, Wp, order, resid, ctl, img_status, st);
  }
  const int W = nP / GR;
  // Left-looking: spreading an image over W workgroups costs a device-scope barrier per step; it pays while the
  // batch leaves most of the device idle.
  if ((long)B * W > 256) {
    hipLaunchKernelGGL(greedy_single_kernel, dim3(B), dim3(TPB), 0, st, G, n, nP, k, Lt, order, resid);
    return hipGetLastError();
  }
  // the workgroups of one image wait for one another, so one image has to fit the device
  static PerDeviceInt cache;
  int capacity = 0;
  const hipError_t ec = resident_workgroups(cache, greedy_kernel, GT, 0, &capacity);
  if (ec != hipSuccess) return ec;
  if (W > capacity) return hipErrorInvalidValue;
  unsigned long long* posts = (unsigned long long*)((char*)scratch + (((size_t)B * sizeof(GreedyCtl) + 255) / 256) * 256);
  hipLaunchKernelGGL(greedy_init_kernel, dim3((B + 255) / 256), dim3(256), 0, st, ctl, B);
  hipLaunchKernelGGL(greedy_kernel, dim3((unsigned)(B * W)), dim3(GT), 0, st, G, n, nP, k, Lt, order, resid, ctl, posts,
                     img_status, barrier_limit_ticks());
  return hipGetLastError();
}

hipError_t launch_greedy_finish(const int32_t* order, const int32_t* idx_m, int B, int M, int k, int32_t* idx_out,
                                int32_t* pick_out, hipStream_t st) {
  if (M > 4096) return hipErrorInvalidValue;
  hipLaunchKernelGGL(greedy_finish_kernel, dim3(B), dim3(TPB), 0, st, order, idx_m, M, k, idx_out, pick_out);
  return hipGetLastError();
}

}  // namespace covspec
