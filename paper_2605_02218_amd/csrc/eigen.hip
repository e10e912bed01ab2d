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
// Parallel form: rows are grouped in blocks of 8; a round-robin tournament pairs the
// blocks, one launch per tournament round, one wave per block pair.  The wave
//   1. forms the 16x16 Gram H = P P^T of its 16 rows with v_mfma_f64_16x16x4 (the A and
//      B operand of that product are the same registers),
//   2. runs one cyclic sweep of two-sided Jacobi rotations on H in LDS, accumulating the
//      16x16 orthogonal W,
//   3. applies P <- W^T P with the same MFMA.
// fp64 MFMA layouts (checked on the device): operand lane l holds (row|col = l%16,
// k = l/16); result lane l, register v holds (row 4v + l/16, col l%16).
#include "common.h"
#include "kernels.h"

namespace covspec {

namespace {

struct JacobiCtl {
  unsigned long long maxoff;  // bits of the largest |cos| between two rows seen in the current sweep
  int done;
  int sweeps;
  double floor2;              // rows with squared norm below this are treated as zero
};

constexpr double kRotEps = 1e-15;   // rotations below this relative size are skipped
constexpr double kConvTol = 1e-9;   // sweep-level convergence: every visited pair below this
constexpr int kMaxSweeps = 14;

__global__ __launch_bounds__(256) void jacobi_init_kernel(const double* __restrict__ A, int n, int nP, JacobiCtl* ctl) {
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
    ctl[b].done = 0;
    ctl[b].sweeps = 0;
    double f = 1e-13 * t;
    ctl[b].floor2 = f * f;
  }
}

__global__ void jacobi_check_kernel(JacobiCtl* ctl, int B) {
  int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  if (!ctl[b].done) {
    ctl[b].sweeps += 1;
    if (__longlong_as_double((long long)ctl[b].maxoff) < kConvTol) ctl[b].done = 1;
  }
  ctl[b].maxoff = 0ull;
}

// circle-method tournament over `np` (even) players: pair `m` of round `rd`
__device__ __forceinline__ void tournament_pair(int np, int rd, int m, int& p, int& q) {
  if (m == 0) { p = np - 1; q = rd; }
  else { p = (rd + m) % (np - 1); q = (rd - m + (np - 1)) % (np - 1); }
}

__global__ __launch_bounds__(64) void jacobi_round_kernel(double* __restrict__ A, int nP, int nb, int round, JacobiCtl* ctl) {
  __shared__ double Hs[16][17];
  __shared__ double Ws[16][17];
  __shared__ double cs_c[8], cs_s[8];
  __shared__ int any_rot;

  const int npairs = nb >> 1;
  const int b = blockIdx.x / npairs, pr = blockIdx.x - b * npairs;
  if (ctl[b].done) return;
  int I, J;
  tournament_pair(nb, round, pr, I, J);
  const int l = threadIdx.x, i16 = l & 15, kq = l >> 4;
  double* Ab = A + (long)b * nP * nP;
  auto grow = [&](int i) -> long { return (i < 8) ? (long)I * 8 + i : (long)J * 8 + (i - 8); };

  // ---- 1. H = P P^T
  {
    const double* rp = Ab + grow(i16) * nP + 4 * kq;
    f64x4_t acc = {0.0, 0.0, 0.0, 0.0};
    for (int c0 = 0; c0 < nP; c0 += 16) {
      f64x4_t a = *(const f64x4_t*)(rp + c0);
#pragma unroll
      for (int t = 0; t < 4; ++t) acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a[t], a[t], acc, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) Hs[4 * v + kq][i16] = acc[v];
    for (int e = l; e < 256; e += 64) Ws[e >> 4][e & 15] = ((e >> 4) == (e & 15)) ? 1.0 : 0.0;
    if (l == 0) any_rot = 0;
  }
  __syncthreads();

  // ---- 2. one cyclic sweep of rotations on H, W <- W J
  const double floor2 = ctl[b].floor2;
  double offmax = 0.0;
  const int m = l >> 3, u = l & 7;
  for (int rd = 0; rd < 15; ++rd) {
    int p, q;
    tournament_pair(16, rd, m, p, q);
    if (u == 0) {
      const double al = Hs[p][p], be = Hs[q][q], ga = Hs[p][q];
      double c = 1.0, s = 0.0;
      if (al > floor2 && be > floor2) {
        const double lim = sqrt(al * be);
        const double aga = fabs(ga);
        offmax = fmax(offmax, aga / lim);
        if (aga > kRotEps * lim) {
          const double zeta = (be - al) / (2.0 * ga);
          const double t = copysign(1.0, zeta) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
          c = 1.0 / sqrt(1.0 + t * t);
          s = c * t;
          any_rot = 1;
        }
      }
      cs_c[m] = c;
      cs_s[m] = s;
    }
    __syncthreads();
    const double c = cs_c[m], s = cs_s[m];
#pragma unroll
    for (int h = 0; h < 2; ++h) {  // rows p,q of H:  J^T H
      const int jj = u + 8 * h;
      const double hp = Hs[p][jj], hq = Hs[q][jj];
      Hs[p][jj] = c * hp - s * hq;
      Hs[q][jj] = s * hp + c * hq;
    }
    __syncthreads();
#pragma unroll
    for (int h = 0; h < 2; ++h) {  // columns p,q of H and W:  (.) J
      const int ii = u + 8 * h;
      const double hp = Hs[ii][p], hq = Hs[ii][q];
      Hs[ii][p] = c * hp - s * hq;
      Hs[ii][q] = s * hp + c * hq;
      const double wp = Ws[ii][p], wq = Ws[ii][q];
      Ws[ii][p] = c * wp - s * wq;
      Ws[ii][q] = s * wp + c * wq;
    }
    __syncthreads();
  }

  // ---- 3. P <- W^T P  (skipped when every rotation of this pair was the identity)
  if (any_rot) {
    double wa[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) wa[t] = Ws[4 * t + kq][i16];
    long rload[4], rstore[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) { rload[t] = grow(4 * t + kq) * nP + i16; rstore[t] = rload[t]; }
    for (int c0 = 0; c0 < nP; c0 += 16) {
      double pb[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) pb[t] = Ab[rload[t] + c0];
      f64x4_t d = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int t = 0; t < 4; ++t) d = __builtin_amdgcn_mfma_f64_16x16x4f64(wa[t], pb[t], d, 0, 0, 0);
#pragma unroll
      for (int v = 0; v < 4; ++v) Ab[rstore[v] + c0] = d[v];
    }
  }
  offmax = wave_max(offmax);
  if (l == 0 && offmax > 0.0) atomicMax(&ctl[b].maxoff, (unsigned long long)__double_as_longlong(offmax));
}

// lam[b*nP + k] = |row k of A[b]|, one wave per row
__global__ __launch_bounds__(256) void row_length_kernel(const double* __restrict__ A, int n, int nP, double* __restrict__ lam) {
  const int lane = threadIdx.x & 63;
  const int k = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int b = blockIdx.y;
  if (k >= n) return;
  const double* row = A + ((long)b * nP + k) * nP;
  double s = 0.0;
  for (int j = lane; j < nP; j += 64) s = fma(row[j], row[j], s);
  s = wave_sum(s);
  if (lane == 0) lam[(long)b * nP + k] = sqrt(s);
}

// c[b,i] = sum_{k in top-r by lam} A[k][i]^2 / lam[k], rows added in ascending k
__global__ __launch_bounds__(256) void energy_kernel(const double* __restrict__ A, int n, int nP, int r,
                                                      const double* __restrict__ lam, float* __restrict__ c) {
  __shared__ double slam[4096];
  __shared__ unsigned char sel[4096];
  const int b = blockIdx.y;
  const double* lb = lam + (long)b * nP;
  for (int k = threadIdx.x; k < n; k += 256) slam[k] = lb[k];
  __syncthreads();
  for (int k = threadIdx.x; k < n; k += 256) {
    const double v = slam[k];
    int rank = 0;
    for (int j = 0; j < n; ++j) {
      const double w = slam[j];
      rank += (w > v || (w == v && j < k)) ? 1 : 0;
    }
    sel[k] = (rank < r && v > 0.0) ? 1 : 0;
  }
  __syncthreads();
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const double* Ab = A + (long)b * nP * nP + i;
  double acc = 0.0;
  for (int k = 0; k < n; ++k) {
    if (sel[k]) {
      const double a = Ab[(long)k * nP];
      acc += a * a / slam[k];
    }
  }
  c[(long)b * n + i] = (float)acc;
}

}  // namespace

size_t jacobi_ctl_bytes(int B) { return sizeof(JacobiCtl) * (size_t)B; }

hipError_t launch_jacobi_eigen(double* A, int B, int n, int nP, void* ctl_, hipStream_t st) {
  if (nP % 16 != 0 || n > nP) return hipErrorInvalidValue;
  JacobiCtl* ctl = (JacobiCtl*)ctl_;
  const int nb = nP / 8;  // even, since nP % 16 == 0
  hipLaunchKernelGGL(jacobi_init_kernel, dim3(B), dim3(256), 0, st, A, n, nP, ctl);
  if (nb >= 2) {
    for (int sweep = 0; sweep < kMaxSweeps; ++sweep) {
      for (int round = 0; round < nb - 1; ++round)
        hipLaunchKernelGGL(jacobi_round_kernel, dim3((unsigned)(B * (nb / 2))), dim3(64), 0, st, A, nP, nb, round, ctl);
      hipLaunchKernelGGL(jacobi_check_kernel, dim3((B + 63) / 64), dim3(64), 0, st, ctl, B);
    }
  }
  return hipGetLastError();
}

hipError_t launch_subspace_energy(const double* A, int B, int n, int nP, int r, double* lam, float* c, hipStream_t st) {
  if (n > 4096) return hipErrorInvalidValue;
  hipLaunchKernelGGL(row_length_kernel, dim3((n + 3) / 4, B), dim3(256), 0, st, A, n, nP, lam);
  hipLaunchKernelGGL(energy_kernel, dim3((n + 255) / 256, B), dim3(256), 0, st, A, n, nP, r, lam, c);
  return hipGetLastError();
}

}  // namespace covspec
