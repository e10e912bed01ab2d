// Rank-r truncated SVD of the pre-selected tokens and their subspace energies
// (paper Sec. III-A.3, SVD and energy equations), via the token Gram matrix.
//
// With Z_M = U S V^T (d x M) the Gram matrix G = Z_M^T Z_M = V S^2 V^T is M x M and
// c_i = sum_{k<r} S_k^2 V_ik^2.  G is diagonalised by a one-sided (Hestenes) block
// Jacobi iteration on its ROWS in fp64: orthogonal row operations A <- J^T A, started
// from A = G, converge to A = L V^T (row k = lambda_k v_k^T, lambda = S^2), because the
// rows of J^T G become mutually orthogonal exactly when J holds the eigenvectors.  Then
// |row k| = lambda_k and c_i = sum over the r longest rows of A_ki^2 / |row k|.
//
// Parallel form: rows are grouped in super-blocks of 32; a round-robin tournament pairs the
// super-blocks, one 512-thread workgroup per pair and image.  The whole solve is ONE launch: the
// workgroups of an image meet at a barrier in global memory after every tournament round.  A
// workgroup takes its (image, slot) from a ticket counter when it starts, so the workgroups that are
// resident always hold the lowest tickets, i.e. whole images plus at most one partial image whose
// missing workgroups are the next to be dispatched once any image finishes; the launcher checks that
// one image fits the device, and every wait is bounded by a wall-clock limit.  In a round the workgroup
//   1. forms the 64x64 Gram H = P P^T of its 64 rows with v_mfma_f64_16x16x4 (waves split the
//      columns, partial tiles are summed in LDS; the A and B operand of a diagonal tile are the
//      same registers),
//   2. runs two-sided Jacobi rotations on H in LDS, accumulating the 64x64 orthogonal W: every
//      cross pair (one row from each super-block) once, or - in the first round of a sweep, which
//      also has to orthogonalise the rows inside a super-block - every pair once,
//   3. applies P <- W^T P with the same MFMA.
// So the 64 x n panel crosses HBM three times per 1024 (or 2016) rotations, and all rotation
// arithmetic runs on LDS-resident data.
// fp64 MFMA layouts (checked on the device): operand lane l holds (row|col = l%16,
// k = l/16); result lane l, register v holds (row 4v + l/16, col l%16).
#include "common.h"
#include "host_cache.h"
#include "kernels.h"

namespace covspec {

namespace {

constexpr int kMaxSweeps = 30;

struct JacobiCtl {
  unsigned long long maxoff[kMaxSweeps + 2];  // per sweep: bits of the largest admixture weight seen (see below)
  ImageBarrier bar;           // barrier of the image's workgroups; bar.failed: a wait ran into its time limit,
                              // the result is invalid (the rows are set to NaN)
  unsigned int ticket;        // ctl[0] only: next (image, slot) to hand to a starting workgroup
  int done;
  int sweeps;
  double floor2;              // rows with squared norm below this are treated as zero
  double long2;               // squared length of the r-th longest row after the previous sweep
};

// Only the r longest rows enter the energies, and they settle many sweeps before the short rows (the
// tail of a graded spectrum) become orthogonal among themselves.  Leaving a pair (p, q) unrotated mixes
// the direction of the longer row with relative weight |cos(p,q)| * (shorter/longer)^2 (the rotation
// angle is ~ gamma / (alpha - beta), and the admixture carries the shorter row's length), so a sweep
// counts as converged when that weight is below kConvTol for every visited pair that holds one of the r
// longest rows; which rows those are is re-measured after every sweep.  The weight is about 40x the
// relative error it leaves in the energies, which are returned in fp32 (6e-8), and the sweep that
// measures it also reduces it, so 3e-7 leaves the energies converged to well below their last bit.
constexpr double kRotEps = 1e-15;   // rotations below this relative size are skipped
constexpr double kConvTol = 3e-7;
// A sweep over ALL pairs that measures a small largest weight w leaves weights of a few w^2 behind (the quadratic
// convergence of the cyclic method; 1 to 4 w^2 on the workloads), so when such a sweep measures less than kEarlyTol
// the sweep after it could only confirm: the solve ends there.  What it leaves in the Ritz residual, 2 to 4 w^2 <=
// 1e-10, is a tenth of what the residual check accepts (with 2e-5 one image of 64 failed that check and paid for a
// second pass).  Banded sweeps do not qualify: they leave the far pairs alone.
constexpr double kEarlyTol = 5e-6;
constexpr double kBandSwitch = 1e-2;   // banded sweeps while the previous sweep's largest weight is above this

__global__ __launch_bounds__(256) void jacobi_init_kernel(const double* __restrict__ A, int n, int nP, JacobiCtl* ctl,
                                                             const int* __restrict__ preset_done) {
  __shared__ double red[4];
  const int b = blockIdx.x;
  const double* Ab = A + (long)b * nP * nP;
  double tr = 0.0;
  for (int i = threadIdx.x; i < n; i += 256) tr += Ab[(long)i * nP + i];
  tr = wave_sum(tr);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = tr;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = red[0] + red[1] + red[2] + red[3];
    for (int k = 0; k < kMaxSweeps + 2; ++k) ctl[b].maxoff[k] = 0ull;
    ctl[b].bar.arrived = 0u;
    ctl[b].bar.failed = 0;
    ctl[b].ticket = 0u;
    ctl[b].done = preset_done ? preset_done[b] : 0;
    ctl[b].sweeps = 0;
    double f = 1e-13 * t;
    ctl[b].floor2 = f * f;
    ctl[b].long2 = 0.0;       // first sweep: every row counts
  }
}

// circle-method tournament over `np` (even) players: pair `m` of round `rd`
__device__ __forceinline__ void tournament_pair(int np, int rd, int m, int& p, int& q) {
  if (m == 0) { p = np - 1; q = rd; }
  else { p = (rd + m) % (np - 1); q = (rd - m + (np - 1)) % (np - 1); }
}

// Banded schedule.  When the matrix is the Rayleigh-Ritz projection of a block iteration, its rows are ordered
// like the eigenvalues and row p only couples to rows whose eigenvalues are near its own: super-blocks more than
// a few apart are orthogonal from the start and stay so (a rotation mixes two rows, so what it feeds into a far
// pair is the product of two small couplings).  A sweep then only visits the pairs (I, I + d), d = 1..dmax, as
// rounds (d, parity): the pairs with (I / d) even, then those with (I / d) odd, each a set of disjoint pairs.
// That is 2 dmax rounds instead of nsb - 1, nearest first, and the sweeps converge at the tournament's rate (CPU
// model on the workloads' matrices).  What the band leaves out is small but not nothing: a short row of the wanted
// set that keeps an admixture delta of a long, far row shows a residual of delta * (long / short), so the banded
// sweeps only do the bulk of the work (while the largest weight seen stays above kBandSwitch) and the solve ends
// with tournament sweeps over all pairs, which also are the ones that decide convergence.
// Pair `m` of round (d, parity); false if there is none.
__device__ __forceinline__ bool band_pair(int nsb, int dist, int parity, int m, int& p, int& q) {
  int seen = 0;
  for (int i = 0; i + dist < nsb; ++i) {
    if (((i / dist) & 1) != parity) continue;
    if (seen == m) { p = i; q = i + dist; return true; }
    ++seen;
  }
  return false;
}

constexpr int SB = 32;        // rows per super-block
constexpr int PR = 2 * SB;    // rows per workgroup
constexpr int HP = PR + 1;    // LDS pitch (doubles)
#ifndef COVSPEC_JACOBI_THREADS
#define COVSPEC_JACOBI_THREADS 512
#endif
constexpr int JT = COVSPEC_JACOBI_THREADS;   // threads per workgroup of the solve: 256 or 512
constexpr int JW = JT / 64;                  // waves
static_assert(JT == 256 || JT == 512, "the visit's index mappings are written for 4 or 8 waves");

// LDS of the solve kernel (file scope: shared by the kernel and the visit function below).
__shared__ double Hs[PR * HP];
__shared__ double Ws[PR * HP];
__shared__ double cs_c[32], cs_s[32];
__shared__ int any_rot;
__shared__ int s_flag;

// One visit of a pair of super-blocks (I, J) of the image whose matrix starts at Ab (steps 1-3 of the header).
// `full`: the rows inside each super-block are paired too (first round of a sweep).  Returns the largest
// admixture weight seen (valid in wave 0).  Kept out of line so that the registers of the three phases are
// allocated for this function alone and not held across the sweep loop of the caller.
__device__ __noinline__ double jacobi_visit(double* Ab, double* len2b, int nP, int I, int J, bool full, double floor2, double long2) {
  const int tid = threadIdx.x, l = tid & 63, w = tid >> 6, i16 = l & 15, kq = l >> 4;
  const int nchunks = nP >> 4;
  auto grow = [&](int i) -> int { return (i < SB) ? I * SB + i : J * SB + (i - SB); };   // nP <= 4096: offsets fit an int

  // ---- 1. H = P P^T : wave w takes column chunks w, w + JW, ...; upper tiles only.  The waves' partial tiles are
  //         added in a fixed order (the result must not depend on which wave comes first): the waves of the lower
  //         half one after the other into Hs, those of the upper half likewise into Ws at the same time, then Hs += Ws.
  for (int e = tid; e < PR * HP; e += JT) { Hs[e] = 0.0; Ws[e] = 0.0; }
  if (tid == 0) any_rot = 0;
  {
    f64x4_t acc[10];
#pragma unroll
    for (int t = 0; t < 10; ++t) acc[t] = (f64x4_t){0.0, 0.0, 0.0, 0.0};
    int rp[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) rp[x] = grow(16 * x + i16) * nP + 4 * kq;
    // the rows were last written by other workgroups, so every load is a long trip: keep two chunks in flight
    f64x4_t f0[4], f1[4], f2[4];
    auto fetch = [&](f64x4_t* f, int c) {
      if (c < nchunks) {
#pragma unroll
        for (int x = 0; x < 4; ++x) f[x] = *(const f64x4_t*)(Ab + rp[x] + 16 * c);
      }
    };
#pragma unroll
    for (int x = 0; x < 4; ++x) f0[x] = f1[x] = f2[x] = (f64x4_t){0.0, 0.0, 0.0, 0.0};
    fetch(f0, w);
    fetch(f1, w + JW);
#pragma unroll 1
    for (int c = w; c < nchunks; c += JW) {
      fetch(f2, c + 2 * JW);
      int t = 0;
#pragma unroll
      for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int y = x; y < 4; ++y) {
#pragma unroll
          for (int k = 0; k < 4; ++k) acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(f0[x][k], f0[y][k], acc[t], 0, 0, 0);
          ++t;
        }
#pragma unroll
      for (int x = 0; x < 4; ++x) { f0[x] = f1[x]; f1[x] = f2[x]; }
    }
    __syncthreads();  // zero fill visible
    double* part = (w < JW / 2) ? Hs : Ws;
    for (int ww = 0; ww < JW / 2; ++ww) {
      if ((w % (JW / 2)) == ww) {
        int t = 0;
#pragma unroll
        for (int x = 0; x < 4; ++x)
#pragma unroll
          for (int y = x; y < 4; ++y) {
#pragma unroll
            for (int v = 0; v < 4; ++v) part[(16 * x + 4 * v + kq) * HP + 16 * y + i16] += acc[t][v];
            ++t;
          }
      }
      __syncthreads();
    }
    for (int e = tid; e < PR * PR; e += JT) {
      const int r = e >> 6, c = e & 63;
      if ((r >> 4) <= (c >> 4)) Hs[r * HP + c] += Ws[r * HP + c];
    }
    __syncthreads();
    // mirror the strictly-upper tiles, identity into W
    for (int e = tid; e < PR * PR; e += JT) {
      const int r = e >> 6, c = e & 63;
      if ((r >> 4) > (c >> 4)) Hs[r * HP + c] = Hs[c * HP + r];
      Ws[r * HP + c] = (r == c) ? 1.0 : 0.0;
    }
    __syncthreads();
  }

  // ---- 2. rotations on H (two-sided), W <- W J
  // A round holds 32 disjoint rotations.  Phase A: 32 threads compute them.  Phase B: the 2x2 block of
  // H at (pair a, pair b) becomes R_a^T H_ab R_b and depends on nothing else, so all 1024 blocks (and the
  // column pairs of W) are updated in place in one pass between two barriers.
  // (floor2, long2: read at the top of the round)
  const int nrounds = full ? PR - 1 : SB;
  double meas2 = 0.0;   // largest squared admixture weight seen by this thread
  // This thread's share of a step: column pair b2 (of H and W), H row pairs a0 + NA*k, W rows a0 + NA*k.
  // The (p, q) of a pair is carried from step to step: circle method (p, q advance by one mod 63; pair 0
  // keeps p = 63) when all 64 rows meet, else p = pair id and q walks cyclically over the second super-block.
  constexpr int NA = JT / 32;        // row-pair groups: thread (b2, a0) takes the row pairs a0, a0 + NA, ...
  constexpr int HB = 32 / NA;        // H blocks per thread and step
  constexpr int WR = 64 / NA;        // W rows per thread and step
  const int b2 = tid & 31, a0 = tid >> 5;
  int pb = full ? (b2 == 0 ? PR - 1 : b2) : b2;
  int qb = full ? (b2 == 0 ? 0 : PR - 1 - b2) : SB + b2;
  int pa[HB], qa[HB];
#pragma unroll
  for (int k = 0; k < HB; ++k) {
    const int m = a0 + NA * k;
    pa[k] = full ? (m == 0 ? PR - 1 : m) : m;
    qa[k] = full ? (m == 0 ? 0 : PR - 1 - m) : SB + m;
  }
  auto advance = [&](int m, int& p_, int& q_) {
    if (full) {
      q_ = (q_ + 1 == PR - 1) ? 0 : q_ + 1;
      if (m != 0) p_ = (p_ + 1 == PR - 1) ? 0 : p_ + 1;
    } else {
      q_ = SB + ((q_ + 1) & (SB - 1));
    }
  };
#pragma unroll 1
  for (int rd = 0; rd < nrounds; ++rd) {
    if (tid < 32) {   // pair id = tid = b2
      const double al = Hs[pb * HP + pb], be = Hs[qb * HP + qb], ga = Hs[pb * HP + qb];
      double c = 1.0, s = 0.0;
      if (al > floor2 && be > floor2) {
        const double g2 = ga * ga, ab = al * be;
        const double hi = fmax(al, be), lo = fmin(al, be);
        if (hi >= long2) {   // weight^2 = (g2 / ab) (lo / hi)^2 = g2 lo / hi^3; a few digits are enough
          const double rh = __builtin_amdgcn_rcp(hi);
          meas2 = fmax(meas2, g2 * lo * rh * rh * rh);
        }
        if (g2 > (kRotEps * kRotEps) * ab) {
          // hardware reciprocal / reciprocal square root estimates, refined by Newton steps: the angle needs
          // few digits, but c^2 + s^2 = 1 has to hold to rounding, so c gets two steps
          const double de = be - al;
          const double x = fma(de, de, 4.0 * g2);
          const double rs = __builtin_amdgcn_rsq(x);
          double rho = x * rs;
          rho = fma(0.5 * rs, fma(-rho, rho, x), rho);
          const double den = de + copysign(rho, de);
          double rd_ = __builtin_amdgcn_rcp(den);
          rd_ = rd_ * fma(-den, rd_, 2.0);
          const double t = 2.0 * ga * rd_;
          const double u = fma(t, t, 1.0);
          c = __builtin_amdgcn_rsq(u);
          c = c * fma(-0.5 * u, c * c, 1.5);
          c = c * fma(-0.5 * u, c * c, 1.5);
          s = c * t;
          any_rot = 1;
        }
      }
      cs_c[tid] = c;
      cs_s[tid] = s;
    }
    __syncthreads();
    {
      // all loads first, then the arithmetic, then all stores: the blocks are disjoint, which the compiler
      // cannot know, and it would otherwise wait out one LDS round trip per block
      const double cb = cs_c[b2], sb = cs_s[b2];
      double ca[HB], sa[HB], h00[HB], h01[HB], h10[HB], h11[HB], wp[WR], wq[WR];
#pragma unroll
      for (int k = 0; k < HB; ++k) {
        ca[k] = cs_c[a0 + NA * k];
        sa[k] = cs_s[a0 + NA * k];
        h00[k] = Hs[pa[k] * HP + pb];
        h01[k] = Hs[pa[k] * HP + qb];
        h10[k] = Hs[qa[k] * HP + pb];
        h11[k] = Hs[qa[k] * HP + qb];
      }
#pragma unroll
      for (int k = 0; k < WR; ++k) {
        wp[k] = Ws[(a0 + NA * k) * HP + pb];
        wq[k] = Ws[(a0 + NA * k) * HP + qb];
      }
#pragma unroll
      for (int k = 0; k < HB; ++k) {   // H block (a0 + NA k, b2) <- R_a^T H R_b
        const double t00 = ca[k] * h00[k] - sa[k] * h10[k], t01 = ca[k] * h01[k] - sa[k] * h11[k];
        const double t10 = sa[k] * h00[k] + ca[k] * h10[k], t11 = sa[k] * h01[k] + ca[k] * h11[k];
        h00[k] = cb * t00 - sb * t01;
        h01[k] = sb * t00 + cb * t01;
        h10[k] = cb * t10 - sb * t11;
        h11[k] = sb * t10 + cb * t11;
      }
#pragma unroll
      for (int k = 0; k < WR; ++k) {   // W columns (pb, qb), row a0 + NA k
        const double x0 = cb * wp[k] - sb * wq[k];
        wq[k] = sb * wp[k] + cb * wq[k];
        wp[k] = x0;
      }
#pragma unroll
      for (int k = 0; k < HB; ++k) {
        Hs[pa[k] * HP + pb] = h00[k];
        Hs[pa[k] * HP + qb] = h01[k];
        Hs[qa[k] * HP + pb] = h10[k];
        Hs[qa[k] * HP + qb] = h11[k];
      }
#pragma unroll
      for (int k = 0; k < WR; ++k) {
        Ws[(a0 + NA * k) * HP + pb] = wp[k];
        Ws[(a0 + NA * k) * HP + qb] = wq[k];
      }
    }
    advance(b2, pb, qb);
#pragma unroll
    for (int k = 0; k < HB; ++k) advance(a0 + NA * k, pa[k], qa[k]);
    __syncthreads();
  }
  // squared row lengths after this visit (the diagonal of the rotated Gram block)
  if (tid < PR) len2b[grow(tid)] = Hs[tid * HP + tid];

  // ---- 3. P <- W^T P  (skipped when every rotation of this pair was the identity)
  if (any_rot) {
    double wa[4][16];   // A operand of k-step t, tile a: W[4t + kq][16a + i16]
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int t = 0; t < 16; ++t) wa[a][t] = Ws[(4 * t + kq) * HP + 16 * a + i16];
    int roff[16];
#pragma unroll
    for (int t = 0; t < 16; ++t) roff[t] = grow(4 * t + kq) * nP + i16;
    for (int c = w; c < nchunks; c += JW) {
      double pb[16];
#pragma unroll
      for (int t = 0; t < 16; ++t) pb[t] = Ab[roff[t] + 16 * c];
      f64x4_t d[4];
#pragma unroll
      for (int a = 0; a < 4; ++a) d[a] = (f64x4_t){0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int t = 0; t < 16; ++t)
#pragma unroll
        for (int a = 0; a < 4; ++a) d[a] = __builtin_amdgcn_mfma_f64_16x16x4f64(wa[a][t], pb[t], d[a], 0, 0, 0);
      // result tile a, register v -> row 16a + 4v + kq = (4*(4a+v) + kq): the load offset of k-step 4a+v
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int v = 0; v < 4; ++v) Ab[roff[4 * a + v] + 16 * c] = d[a][v];
    }
  }
  return wave_max(meas2);
}

// The whole solve of all images: workgroup (image b, slot pr) visits the pair `pr` of every tournament round
// of every sweep; after a sweep, slot 0 decides convergence and re-measures which rows are the r longest.
// A and len2 are written and re-read by different workgroups between barriers, hence no __restrict__.
__global__ __launch_bounds__(JT) void jacobi_solve_kernel(double* A, int n, int nP, int nsb, int r, JacobiCtl* ctl, double* len2,
                                                              const int* __restrict__ band, int* img_status, long long limit_ticks) {
  const int npairs = nsb >> 1;
  const int tid = threadIdx.x;
  if (tid == 0) s_flag = (int)atomicAdd(&ctl[0].ticket, 1u);
  __syncthreads();
  const int ticket = s_flag;
  __syncthreads();   // s_flag is reused by the barriers
  const int b = ticket / npairs, pr = ticket - b * npairs;
  JacobiCtl* cb = ctl + b;
  if (cb->done) return;   // set before the launch, so the same for every workgroup of the image
  double* Ab = A + (long)b * nP * nP;
  double* len2b = len2 + (long)b * nP;
  const double floor2 = cb->floor2;   // written by the init kernel
  unsigned int target = 0;
  bool alive = true;
  // largest super-block distance that is visited (written before the launch); the banded schedule is taken when it
  // has fewer rounds than the tournament
  const int dmax = band ? band[b] : 0;
  const bool may_band = dmax >= 1 && 2 * dmax < nsb - 1;

#pragma unroll 1
  for (int sweep = 0; sweep < kMaxSweeps && alive; ++sweep) {
    const double long2 = __hip_atomic_load(&cb->long2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // the previous sweep's largest weight: complete behind the barrier that closed that sweep, the same in every workgroup
    const double prev = sweep == 0 ? 1.0
                                   : __longlong_as_double((long long)__hip_atomic_load(&cb->maxoff[sweep - 1], __ATOMIC_RELAXED,
                                                                                        __HIP_MEMORY_SCOPE_AGENT));
    const bool banded = may_band && prev > kBandSwitch;
    const int nrounds = banded ? 2 * dmax : nsb - 1;
#pragma unroll 1
    for (int round = 0; round < nrounds && alive; ++round) {
      int I = 0, J = 0;
      bool have = true;
      if (banded) {
        if (!band_pair(nsb, (round >> 1) + 1, round & 1, 0, I, J)) continue;   // a round without pairs (the same for every workgroup)
        have = band_pair(nsb, (round >> 1) + 1, round & 1, pr, I, J);
      } else {
        tournament_pair(nsb, round, pr, I, J);
      }
      if (have) {
        // the rows inside a super-block are paired in the first round of a sweep, in which every super-block takes part
        const double meas = jacobi_visit(Ab, len2b, nP, I, J, round == 0, floor2, long2);
        if (tid == 0 && meas > 0.0) atomicMax(&cb->maxoff[sweep], (unsigned long long)__double_as_longlong(sqrt(meas)));
      }
      target += npairs;
      alive = image_barrier_wait(&cb->bar, target, &s_flag, limit_ticks);
    }
    if (!alive) break;
    // ---- end of the sweep: slot 0 decides convergence and finds the squared length of the r-th longest row
    if (pr == 0) {
      double* l2 = Hs;   // 4096 doubles fit
      for (int k = tid; k < n; k += JT) l2[k] = len2b[k];
      __syncthreads();
      for (int k = tid; k < n; k += JT) {
        const double v = l2[k];
        int rank = 0;
        for (int j = 0; j < n; ++j) {
          const double u = l2[j];
          rank += (u > v || (u == v && j < k)) ? 1 : 0;
        }
        if (rank == r - 1) __hip_atomic_store(&cb->long2, v * (1.0 - 1e-12), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      if (tid == 0) {
        cb->sweeps = sweep + 1;
        const unsigned long long m = __hip_atomic_load(&cb->maxoff[sweep], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const double mw = __longlong_as_double((long long)m);
        if (mw < kConvTol || (!banded && mw < kEarlyTol)) __hip_atomic_store(&cb->done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    target += npairs;
    alive = image_barrier_wait(&cb->bar, target, &s_flag, limit_ticks);
    if (alive && __hip_atomic_load(&cb->done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) break;
  }
  if (!alive) {
    // a wait ran out: poison this slot's share of the rows so that nothing downstream passes for a result
    const double qnan = __longlong_as_double(0x7ff8000000000000LL);
    for (long e = tid; e < (long)PR * nP; e += JT) Ab[(long)pr * PR * nP + e] = qnan;
    if (img_status && tid == 0) img_status[b] = 1;
  }
}

// dmax[b] = the largest super-block distance d at which two rows of the symmetric matrix H[b] still couple: S[b] = H[b]^2
// is the Gram matrix of the rows of H[b] (the rows the solve rotates), and a pair (p, q) couples with the weight the
// solve measures, |S_pq| sqrt(min(S_pp, S_qq)) / max(S_pp, S_qq)^1.5.  Distances whose largest weight is below `tol`
// are left out (at least 1 is returned).  One workgroup per image; n x n, pitch n, only the lower triangle of S is read.
__global__ __launch_bounds__(1024) void band_limit_kernel(const double* __restrict__ S, int n, double tol, int* __restrict__ dmax,
                                                          const int* __restrict__ skip) {
  __shared__ double diag[4096];
  __shared__ int far;
  const int b = blockIdx.x;
  if (skip && skip[b]) return;     // the solve leaves this image alone
  const double* Sb = S + (long)b * n * n;
  for (int k = threadIdx.x; k < n; k += 1024) diag[k] = Sb[(long)k * n + k];
  if (threadIdx.x == 0) far = 1;
  __syncthreads();
  int mine = 1;
  for (long e = threadIdx.x; e < (long)n * n; e += 1024) {
    const int p = (int)(e / n), q = (int)(e - (long)p * n);
    const int dist = p / SB - q / SB;
    if (dist <= mine) continue;          // also skips the upper triangle and what is already known to couple
    const double a = diag[p], c = diag[q], hi = fmax(a, c), lo = fmin(a, c);
    if (!(lo > 0.0)) continue;
    const double w = fabs(Sb[e]) * sqrt(lo) / (hi * sqrt(hi));
    if (!(w < tol)) mine = dist;         // NaN counts as coupled
  }
  if (mine > 1) atomicMax(&far, mine);
  __syncthreads();
  if (threadIdx.x == 0) dmax[b] = far;
}

// lam[b*rows + k] = |row k of A[b]| (A[b] starts at b*img_stride and has `rows` rows of `pitch`), one wave per row
__global__ __launch_bounds__(256) void row_length_kernel(const double* __restrict__ A, int rows, int pitch, long img_stride,
                                                          double* __restrict__ lam) {
  const int lane = threadIdx.x & 63;
  const int k = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int b = blockIdx.y;
  if (k >= rows) return;
  const double* row = A + b * img_stride + (long)k * pitch;
  double s = 0.0;
  for (int j = lane; j < pitch; j += 64) s = fma(row[j], row[j], s);
  s = wave_sum(s);
  if (lane == 0) lam[(long)b * rows + k] = sqrt(s);
}

// c[b,i] = sum over the r longest rows k of A[b] (rows x pitch) of A[k][i]^2 / |row k|, rows added in
// ascending k; i < n.  Images with (flag[b] != 0) != (run_if != 0) are skipped (flag == nullptr: none).
__global__ __launch_bounds__(256) void energy_kernel(const double* __restrict__ A, int rows, int n, int pitch, long img_stride,
                                                      int r, const double* __restrict__ lam, float* __restrict__ c,
                                                      const int* __restrict__ flag, int run_if) {
  __shared__ double slam[4096];
  __shared__ unsigned char sel[4096];
  const int b = blockIdx.y;
  if (flag && (flag[b] != 0) != (run_if != 0)) return;     // flag: 0 = not converged, any other value = converged
  const double* lb = lam + (long)b * rows;
  for (int k = threadIdx.x; k < rows; k += 256) slam[k] = lb[k];
  __syncthreads();
  for (int k = threadIdx.x; k < rows; k += 256) {
    const double v = slam[k];
    int rank = 0;
    for (int j = 0; j < rows; ++j) {
      const double w = slam[j];
      rank += (w > v || (w == v && j < k)) ? 1 : 0;
    }
    sel[k] = (rank < r && v > 0.0) ? 1 : 0;
  }
  __syncthreads();
  // the selected rows' reciprocal lengths in place of the lengths: a row then costs a thread one load and two
  // multiplications, eight rows' loads in flight (a division per row and one load at a time took 67 us for workload 5)
  for (int k = threadIdx.x; k < rows; k += 256) slam[k] = sel[k] ? 1.0 / slam[k] : 0.0;
  __syncthreads();
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const double* Ab = A + b * img_stride + i;
  double acc = 0.0;
  int k = 0;
  for (; k + 8 <= rows; k += 8) {
    double a[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) a[u] = Ab[(long)(k + u) * pitch];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += sel[k + u] ? a[u] * a[u] * slam[k + u] : 0.0;    // an unselected row may hold anything
  }
  for (; k < rows; ++k) {
    const double a = Ab[(long)k * pitch];
    acc += sel[k] ? a * a * slam[k] : 0.0;
  }
  c[(long)b * n + i] = (float)acc;
}

}  // namespace

size_t jacobi_ctl_bytes(int B) { return sizeof(JacobiCtl) * (size_t)B; }
int jacobi_pitch(int n) { return (n + PR - 1) / PR * PR; }

namespace {
std::atomic<long long> g_barrier_limit{kBarrierLimitTicks};
}
void set_barrier_limit_ticks(long long ticks) { g_barrier_limit.store(ticks > 0 ? ticks : kBarrierLimitTicks); }
long long barrier_limit_ticks() { return g_barrier_limit.load(); }

hipError_t launch_jacobi_eigen(double* A, int B, int n, int nP, int r, void* ctl_, double* len2, const int* preset_done,
                               const int* band, int* img_status, hipStream_t st) {
  if (nP % 64 != 0 || n > nP || n > 4096 || r < 1 || r > n) return hipErrorInvalidValue;
  JacobiCtl* ctl = (JacobiCtl*)ctl_;
  const int nsb = nP / SB;  // even, since nP % 64 == 0
  const int npairs = nsb / 2;
  // the workgroups of one image wait for one another, so one image has to fit the device
  static PerDeviceInt cache;
  int capacity = 0;
  const hipError_t ec = resident_workgroups(cache, jacobi_solve_kernel, JT, 0, &capacity);
  if (ec != hipSuccess) return ec;
  if (npairs > capacity) return hipErrorInvalidValue;
  hipLaunchKernelGGL(jacobi_init_kernel, dim3(B), dim3(256), 0, st, A, n, nP, ctl, preset_done);
  hipLaunchKernelGGL(jacobi_solve_kernel, dim3((unsigned)(B * npairs)), dim3(JT), 0, st, A, n, nP, nsb, r, ctl, len2,
                     band, img_status, barrier_limit_ticks());
  return hipGetLastError();
}

hipError_t launch_band_limit(const double* S, int B, int n, double tol, int* dmax, const int* skip, hipStream_t st) {
  if (n > 4096 || n % SB != 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(band_limit_kernel, dim3(B), dim3(1024), 0, st, S, n, tol, dmax, skip);
  return hipGetLastError();
}

hipError_t launch_row_lengths(const double* A, int B, int rows, int pitch, long img_stride, double* lam, hipStream_t st) {
  hipLaunchKernelGGL(row_length_kernel, dim3((rows + 3) / 4, B), dim3(256), 0, st, A, rows, pitch, img_stride, lam);
  return hipGetLastError();
}

hipError_t launch_subspace_energy(const double* A, int B, int rows, int n, int pitch, long img_stride, int r, double* lam,
                                  float* c, const int* flag, int run_if, hipStream_t st) {
  if (rows > 4096 || r > rows) return hipErrorInvalidValue;
  hipLaunchKernelGGL(row_length_kernel, dim3((rows + 3) / 4, B), dim3(256), 0, st, A, rows, pitch, img_stride, lam);
  hipLaunchKernelGGL(energy_kernel, dim3((n + 255) / 256, B), dim3(256), 0, st, A, rows, n, pitch, img_stride, r, lam, c, flag, run_if);
  return hipGetLastError();
}

}  // namespace covspec
