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
// super-blocks, one launch per tournament round, one 256-thread workgroup per pair.  The workgroup
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
#include "kernels.h"

namespace covspec {

namespace {

struct JacobiCtl {
  unsigned long long maxoff;  // bits of the largest admixture weight seen in the current sweep (see below)
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
constexpr int kMaxSweeps = 30;

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
    ctl[b].maxoff = 0ull;
    ctl[b].done = preset_done ? preset_done[b] : 0;
    ctl[b].sweeps = 0;
    double f = 1e-13 * t;
    ctl[b].floor2 = f * f;
    ctl[b].long2 = 0.0;       // first sweep: every row counts
  }
}

// End of a sweep, one workgroup per image: decide convergence, then find the squared length of the r-th
// longest row from the lengths the round kernels left behind.
__global__ __launch_bounds__(256) void jacobi_check_kernel(const double* __restrict__ len2g, int n, int nP, int r, JacobiCtl* ctl) {
  __shared__ double len2[4096];
  const int b = blockIdx.x;
  if (ctl[b].done) return;
  for (int k = threadIdx.x; k < n; k += 256) len2[k] = len2g[(long)b * nP + k];
  __syncthreads();
  for (int k = threadIdx.x; k < n; k += 256) {
    const double v = len2[k];
    int rank = 0;
    for (int j = 0; j < n; ++j) {
      const double u = len2[j];
      rank += (u > v || (u == v && j < k)) ? 1 : 0;
    }
    if (rank == r - 1) ctl[b].long2 = v * (1.0 - 1e-12);
  }
  if (threadIdx.x == 0) {
    ctl[b].sweeps += 1;
    if (__longlong_as_double((long long)ctl[b].maxoff) < kConvTol) ctl[b].done = 1;
    ctl[b].maxoff = 0ull;
  }
}

// circle-method tournament over `np` (even) players: pair `m` of round `rd`
__device__ __forceinline__ void tournament_pair(int np, int rd, int m, int& p, int& q) {
  if (m == 0) { p = np - 1; q = rd; }
  else { p = (rd + m) % (np - 1); q = (rd - m + (np - 1)) % (np - 1); }
}

constexpr int SB = 32;        // rows per super-block
constexpr int PR = 2 * SB;    // rows per workgroup
constexpr int HP = PR + 1;    // LDS pitch (doubles)

__global__ __launch_bounds__(256, 2) void jacobi_round_kernel(double* __restrict__ A, int nP, int nsb, int round, JacobiCtl* ctl,
                                                              double* __restrict__ len2) {
  __shared__ double Hs[PR * HP];
  __shared__ double Ws[PR * HP];
  __shared__ double cs_c[32], cs_s[32];
  __shared__ int any_rot;

  const int npairs = nsb >> 1;
  const int b = blockIdx.x / npairs, pr = blockIdx.x - b * npairs;
  if (ctl[b].done) return;
  int I, J;
  tournament_pair(nsb, round, pr, I, J);
  const int tid = threadIdx.x, l = tid & 63, w = tid >> 6, i16 = l & 15, kq = l >> 4;
  double* Ab = A + (long)b * nP * nP;
  auto grow = [&](int i) -> long { return (i < SB) ? (long)I * SB + i : (long)J * SB + (i - SB); };
  const int nchunks = nP >> 4;

  // ---- 1. H = P P^T : wave w takes column chunks w, w+4, ...; upper tiles only
  for (int e = tid; e < PR * HP; e += 256) { Hs[e] = 0.0; Ws[e] = 0.0; }
  if (tid == 0) any_rot = 0;
  {
    f64x4_t acc[10];
#pragma unroll
    for (int t = 0; t < 10; ++t) acc[t] = (f64x4_t){0.0, 0.0, 0.0, 0.0};
    const double* rp[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) rp[x] = Ab + grow(16 * x + i16) * nP + 4 * kq;
    for (int c = w; c < nchunks; c += 4) {
      f64x4_t f[4];
#pragma unroll
      for (int x = 0; x < 4; ++x) f[x] = *(const f64x4_t*)(rp[x] + 16 * c);
      int t = 0;
#pragma unroll
      for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int y = x; y < 4; ++y) {
#pragma unroll
          for (int k = 0; k < 4; ++k) acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(f[x][k], f[y][k], acc[t], 0, 0, 0);
          ++t;
        }
    }
    __syncthreads();  // zero fill visible
    for (int ww = 0; ww < 4; ++ww) {
      if (w == ww) {
        int t = 0;
#pragma unroll
        for (int x = 0; x < 4; ++x)
#pragma unroll
          for (int y = x; y < 4; ++y) {
#pragma unroll
            for (int v = 0; v < 4; ++v) Hs[(16 * x + 4 * v + kq) * HP + 16 * y + i16] += acc[t][v];
            ++t;
          }
      }
      __syncthreads();
    }
    // mirror the strictly-upper tiles, identity into W
    for (int e = tid; e < PR * PR; e += 256) {
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
  const double floor2 = ctl[b].floor2, long2 = ctl[b].long2;
  const bool full = (round == 0);
  const int nrounds = full ? PR - 1 : SB;
  double meas2 = 0.0;   // largest squared admixture weight seen by this thread
  auto pair_of = [&](int rd, int m, int& p, int& q) {
    if (full) tournament_pair(PR, rd, m, p, q);
    else { p = m; q = SB + ((m + rd) & (SB - 1)); }
  };
  for (int rd = 0; rd < nrounds; ++rd) {
    if (tid < 32) {
      int p, q;
      pair_of(rd, tid, p, q);
      const double al = Hs[p * HP + p], be = Hs[q * HP + q], ga = Hs[p * HP + q];
      double c = 1.0, s = 0.0;
      if (al > floor2 && be > floor2) {
        const double g2 = ga * ga, ab = al * be;
        const double hi = fmax(al, be), lo = fmin(al, be);
        if (hi >= long2) {
          const double rr = lo / hi;
          meas2 = fmax(meas2, (g2 / ab) * rr * rr);
        }
        if (g2 > (kRotEps * kRotEps) * ab) {
          const double de = be - al;
          const double rho = sqrt(de * de + 4.0 * g2);
          const double t = 2.0 * ga / (de + copysign(rho, de));
          c = 1.0 / sqrt(1.0 + t * t);
          s = c * t;
          any_rot = 1;
        }
      }
      cs_c[tid] = c;
      cs_s[tid] = s;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4; ++k) {   // H blocks (a, b2)
      const int e = tid + 256 * k, a = e >> 5, b2 = e & 31;
      const double ca = cs_c[a], sa = cs_s[a], cb = cs_c[b2], sb = cs_s[b2];
      if (sa != 0.0 || sb != 0.0) {
        int pa, qa, pb, qb;
        pair_of(rd, a, pa, qa);
        pair_of(rd, b2, pb, qb);
        const double h00 = Hs[pa * HP + pb], h01 = Hs[pa * HP + qb], h10 = Hs[qa * HP + pb], h11 = Hs[qa * HP + qb];
        const double t00 = ca * h00 - sa * h10, t01 = ca * h01 - sa * h11;   // R_a^T H
        const double t10 = sa * h00 + ca * h10, t11 = sa * h01 + ca * h11;
        Hs[pa * HP + pb] = cb * t00 - sb * t01;                               // (.) R_b
        Hs[pa * HP + qb] = sb * t00 + cb * t01;
        Hs[qa * HP + pb] = cb * t10 - sb * t11;
        Hs[qa * HP + qb] = sb * t10 + cb * t11;
      }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {   // W column pairs (row i, pair b2)
      const int e = tid + 256 * k, i = e >> 5, b2 = e & 31;
      const double cb = cs_c[b2], sb = cs_s[b2];
      if (sb != 0.0) {
        int pb, qb;
        pair_of(rd, b2, pb, qb);
        const double wp = Ws[i * HP + pb], wq = Ws[i * HP + qb];
        Ws[i * HP + pb] = cb * wp - sb * wq;
        Ws[i * HP + qb] = sb * wp + cb * wq;
      }
    }
    __syncthreads();
  }
  // squared row lengths after this visit (the diagonal of the rotated Gram block)
  if (tid < PR) len2[(long)b * nP + grow(tid)] = Hs[tid * HP + tid];

  // ---- 3. P <- W^T P  (skipped when every rotation of this pair was the identity)
  if (any_rot) {
    double wa[4][16];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int t = 0; t < 16; ++t) wa[a][t] = Ws[(4 * t + kq) * HP + 16 * a + i16];
    long roff[16];
#pragma unroll
    for (int t = 0; t < 16; ++t) roff[t] = grow(4 * t + kq) * nP + i16;
    for (int c = w; c < nchunks; c += 4) {
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
  meas2 = wave_max(meas2);   // only wave 0 holds non-zero values
  if (tid == 0 && meas2 > 0.0) atomicMax(&ctl[b].maxoff, (unsigned long long)__double_as_longlong(sqrt(meas2)));
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
// ascending k; i < n.  Images with flag[b] != run_if are skipped (flag == nullptr: none).
__global__ __launch_bounds__(256) void energy_kernel(const double* __restrict__ A, int rows, int n, int pitch, long img_stride,
                                                      int r, const double* __restrict__ lam, float* __restrict__ c,
                                                      const int* __restrict__ flag, int run_if) {
  __shared__ double slam[4096];
  __shared__ unsigned char sel[4096];
  const int b = blockIdx.y;
  if (flag && flag[b] != run_if) return;
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
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const double* Ab = A + b * img_stride + i;
  double acc = 0.0;
  for (int k = 0; k < rows; ++k) {
    if (sel[k]) {
      const double a = Ab[(long)k * pitch];
      acc += a * a / slam[k];
    }
  }
  c[(long)b * n + i] = (float)acc;
}

}  // namespace

size_t jacobi_ctl_bytes(int B) { return sizeof(JacobiCtl) * (size_t)B; }
int jacobi_pitch(int n) { return (n + PR - 1) / PR * PR; }
int jacobi_launches(int n) { return kMaxSweeps * (jacobi_pitch(n) / SB - 1); }

hipError_t launch_jacobi_eigen(double* A, int B, int n, int nP, int r, void* ctl_, double* len2, const int* preset_done,
                               hipStream_t st) {
  if (nP % 64 != 0 || n > nP || n > 4096 || r < 1 || r > n) return hipErrorInvalidValue;
  JacobiCtl* ctl = (JacobiCtl*)ctl_;
  const int nsb = nP / SB;  // even, since nP % 64 == 0
  hipLaunchKernelGGL(jacobi_init_kernel, dim3(B), dim3(256), 0, st, A, n, nP, ctl, preset_done);
  for (int sweep = 0; sweep < kMaxSweeps; ++sweep) {
    for (int round = 0; round < nsb - 1; ++round)
      hipLaunchKernelGGL(jacobi_round_kernel, dim3((unsigned)(B * (nsb / 2))), dim3(256), 0, st, A, nP, nsb, round, ctl, len2);
    hipLaunchKernelGGL(jacobi_check_kernel, dim3(B), dim3(256), 0, st, len2, n, nP, r, ctl);
  }
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
