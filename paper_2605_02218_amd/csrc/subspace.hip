// Top-r eigen-subspace of the token Gram matrix by block subspace iteration
// (the rank-r truncated SVD of paper Sec. III-A.3 only needs V_r and Sigma_r).
//
// Only the r dominant eigenpairs of G = Z_M^T Z_M enter the energies, so instead of
// diagonalising all of G, a block of P > r vectors is iterated:
//     Y <- G Y,  Y <- orthonormalise(Y)          (P ~ 2r; error shrinks by lambda_{P+1}/lambda_r per step)
// and the r dominant Ritz pairs of the P x P projection Q^T G Q are taken (Rayleigh-Ritz, solved by
// the block Jacobi kernel).  All products are fp64 MFMA GEMMs; the cost scales with r, not with M.
//
// Storage is transposed (vectors are rows, Yt is P x nP) so that every product is in the
// K-contiguous "NT" form of the GEMM kernel: (G Y)^T = Yt G^T = Yt G.
// Orthonormalisation is Cholesky-QR: S = Yt Yt^T = L L^T (blocked right-looking Cholesky, 64-wide
// panels, trailing update on the MFMA), Yt <- L^-1 Yt (blocked forward substitution).
// The start block is Omega G with a fixed +-1 pattern Omega, so exact duplicate tokens (equal rows of
// G) cannot make it rank deficient.
// After the Ritz step the residuals |G u - theta u| of the r dominant Ritz pairs are checked; images
// that fail (slow decay, P too small) fall back to the full block Jacobi solve of G.
#include "common.h"
#include "kernels.h"

namespace covspec {

namespace {

constexpr int NB = 64;        // panel width of Cholesky / substitution
constexpr int NBP = NB + 1;   // LDS pitch

__global__ void omega_kernel(double* __restrict__ om, int P, int n, int nP) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long)P * nP) return;
  const int r = (int)(i / nP), c = (int)(i - (long)r * nP);
  uint32_t h = (uint32_t)r * 0x9E3779B1u ^ ((uint32_t)c + 0x7F4A7C15u) * 0x85EBCA77u;
  h ^= h >> 15; h *= 0x2C1B3C6Du; h ^= h >> 12; h *= 0x297A2D39u; h ^= h >> 15;
  om[i] = (c < n) ? ((h & 1u) ? 1.0 : -1.0) : 0.0;
}

// in-LDS Cholesky of a 64x64 SPD block held in a[NB][NBP] (lower triangle valid on return), 256 threads
__device__ void potrf64_lds(double* a, double floor_) {
  const int tid = threadIdx.x;
  for (int k = 0; k < NB; ++k) {
    if (tid == 0) a[k * NBP + k] = sqrt(fmax(a[k * NBP + k], floor_));
    __syncthreads();
    const double d = a[k * NBP + k];
    if (tid > k && tid < NB) a[tid * NBP + k] /= d;
    __syncthreads();
    // trailing update of the lower triangle: (i, j), k < j <= i < 64
    const int m = NB - 1 - k;                 // remaining order
    for (int e = tid; e < m * m; e += 256) {
      const int i = k + 1 + e / m, j = k + 1 + e % m;
      if (j <= i) a[i * NBP + j] -= a[i * NBP + k] * a[j * NBP + k];
    }
    __syncthreads();
  }
}

// Step J of the blocked Cholesky of S[b] (P x P, pitch P): every workgroup factors the diagonal block
// S[J,J] in LDS (redundantly - it is small), workgroup 0 of an image stores the factor in D[b][J], and
// each thread solves one row of the panel below:  X L_JJ^T = S[I,J]  (in place).
__global__ __launch_bounds__(256) void chol_step_kernel(double* __restrict__ S, double* __restrict__ D, int P, int J,
                                                         int wg_per_image, const int* __restrict__ skip) {
  __shared__ double a[NB * NBP];
  const int b = blockIdx.x / wg_per_image, w = blockIdx.x - b * wg_per_image;
  if (skip && skip[b]) return;
  double* Sb = S + (long)b * P * P;
  const int tid = threadIdx.x;
  const int j0 = J * NB;
  double tr = 0.0;
  for (int e = tid; e < NB * NB; e += 256) {
    const int i = e >> 6, j = e & 63;
    a[i * NBP + j] = Sb[(long)(j0 + i) * P + j0 + j];
  }
  __syncthreads();
  for (int i = 0; i < NB; ++i) tr += a[i * NBP + i];          // same value in every thread
  potrf64_lds(a, 1e-300 + 1e-28 * tr);
  if (w == 0) {
    double* Db = D + ((long)b * (P / NB) + J) * NB * NB;
    for (int e = tid; e < NB * NB; e += 256) {
      const int i = e >> 6, j = e & 63;
      Db[e] = (j <= i) ? a[i * NBP + j] : 0.0;
    }
  }
  const int row = (J + 1) * NB + w * 256 + tid;
  if (row < P) {
    double* x = Sb + (long)row * P + j0;
    double v[NB];
#pragma unroll
    for (int k = 0; k < NB; ++k) v[k] = x[k];
#pragma unroll
    for (int k = 0; k < NB; ++k) {
      double s = v[k];
#pragma unroll
      for (int m = 0; m < k; ++m) s -= v[m] * a[k * NBP + m];
      v[k] = s / a[k * NBP + k];
    }
#pragma unroll
    for (int k = 0; k < NB; ++k) x[k] = v[k];
  }
}

// Yt[b][bi*64 .. +63][:] <- D[b][bi]^-1 Yt[...]: one thread per column, forward substitution
__global__ __launch_bounds__(256) void solve64_kernel(double* __restrict__ Yt, const double* __restrict__ D, int P, int nP,
                                                       int bi, int wg_per_image, const int* __restrict__ skip) {
  __shared__ double a[NB * NBP];
  const int b = blockIdx.x / wg_per_image, w = blockIdx.x - b * wg_per_image;
  if (skip && skip[b]) return;
  const double* Db = D + ((long)b * (P / NB) + bi) * NB * NB;
  for (int e = threadIdx.x; e < NB * NB; e += 256) a[(e >> 6) * NBP + (e & 63)] = Db[e];
  __syncthreads();
  const int col = w * 256 + threadIdx.x;
  if (col >= nP) return;
  double* y = Yt + ((long)b * P + (long)bi * NB) * nP + col;
  double v[NB];
#pragma unroll
  for (int k = 0; k < NB; ++k) v[k] = y[(long)k * nP];
#pragma unroll
  for (int k = 0; k < NB; ++k) {
    double s = v[k];
#pragma unroll
    for (int m = 0; m < k; ++m) s -= a[k * NBP + m] * v[m];
    v[k] = s / a[k * NBP + k];
  }
#pragma unroll
  for (int k = 0; k < NB; ++k) y[(long)k * nP] = v[k];
}

// Residual check of the r dominant Ritz pairs.  Ut rows are theta_k u_k^T, Rt = Ut G.  ok[b] = 1 when
// |Rt_k - theta_k Ut_k| <= tol * theta_k^2 for each of them (theta_k = |Ut_k|, so this is the relative
// residual |G u - theta u| / theta).
__global__ __launch_bounds__(256) void ritz_check_kernel(const double* __restrict__ Ut, const double* __restrict__ Rt,
                                                          const double* __restrict__ lam, int P, int n, int nP, int r,
                                                          double tol, int* __restrict__ ok) {
  __shared__ double slam[4096];
  __shared__ unsigned char sel[4096];
  __shared__ int bad;
  const int b = blockIdx.x, lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const double* lb = lam + (long)b * P;
  for (int k = threadIdx.x; k < P; k += 256) slam[k] = lb[k];
  if (threadIdx.x == 0) bad = 0;
  __syncthreads();
  for (int k = threadIdx.x; k < P; k += 256) {
    const double v = slam[k];
    int rank = 0;
    for (int j = 0; j < P; ++j) { const double u = slam[j]; rank += (u > v || (u == v && j < k)) ? 1 : 0; }
    sel[k] = rank < r;
  }
  __syncthreads();
  for (int k = w; k < P; k += 4) {
    if (!sel[k]) continue;
    const double th = slam[k];
    const double* u = Ut + ((long)b * P + k) * nP;
    const double* rr = Rt + ((long)b * P + k) * nP;
    double s = 0.0;
    for (int j = lane; j < n; j += 64) { const double d = rr[j] - th * u[j]; s = fma(d, d, s); }
    s = wave_sum(s);
    if (lane == 0 && !(sqrt(s) <= tol * th * th)) bad = 1;   // also catches NaN
  }
  __syncthreads();
  if (threadIdx.x == 0) ok[b] = bad ? 0 : 1;
}

}  // namespace

int subspace_block(int n, int r) {
  // P = max(2r, r + 64) rounded up to the panel width; 0 = not worthwhile (P would be most of n)
  int P = 2 * r > r + 64 ? 2 * r : r + 64;
  P = (P + NB - 1) / NB * NB;
  return (4 * P <= 3 * n) ? P : 0;
}

size_t subspace_workspace_bytes(int B, int n, int nP, int P) {
  if (P <= 0) return 0;
  const size_t blk = (size_t)B * P * nP * 8;
  return 2 * blk + (size_t)P * nP * 8 + 2 * (size_t)B * P * P * 8 + (size_t)B * P * NB * 8 + (size_t)B * P * 8 + 1024 + (size_t)B * 4;
}

// Runs the iteration on G[b] (n x n, pitch nP, untouched).  On return, for images with ok[b] = 1, rows
// k of (*ut)[b] (P rows, pitch nP, inside ws) are theta_k u_k^T with the r longest rows converged.
int subspace_product_launches(int iters) { return iters + 2; }   // start block, one per iteration, residuals

hipError_t launch_subspace_eigen(const double* G, int B, int n, int nP, int r, int P, int iters, void* ws_, void* jacobi_ctl,
                                 double* jacobi_len2, int* ok, const double** ut, hipEvent_t probe_begin, hipEvent_t probe_end,
                                 hipStream_t st) {
  if (P <= 0 || P % NB != 0 || P > n || P > 4096) return hipErrorInvalidValue;
  char* ws = (char*)ws_;
  const size_t blk = (size_t)B * P * nP * 8;
  double* Yt = (double*)ws;                 // after the call: Ut
  double* Zt = (double*)(ws + blk);
  double* Om = (double*)(ws + 2 * blk);
  double* S = (double*)(ws + 2 * blk + (size_t)P * nP * 8);
  double* H = S + (size_t)B * P * P;
  double* D = H + (size_t)B * P * P;
  double* lam = D + (size_t)B * P * NB;
  const int nblk = P / NB;
  hipError_t e;

  auto gemm_yt_g = [&](const double* X, double* out) {   // out = X G  (P x nP)
    GemmArgs g;
    g.A = X; g.B = G; g.C = out; g.M = P; g.N = nP; g.K = nP; g.lda = nP; g.ldb = nP; g.ldc = nP;
    g.batch = B; g.strideA = (long)P * nP; g.strideB = (long)nP * nP; g.strideC = (long)P * nP;
    g.epilogue = EPI_STORE_F64;
    return launch_gemm64_nt(g, true, true, st);
  };
  auto cholqr = [&](double* X) -> hipError_t {           // X <- L^-1 X with X X^T = L L^T
    GemmArgs g;
    g.A = X; g.B = X; g.C = S; g.M = P; g.N = P; g.K = nP; g.lda = nP; g.ldb = nP; g.ldc = P;
    g.batch = B; g.strideA = (long)P * nP; g.strideB = (long)P * nP; g.strideC = (long)P * P;
    g.epilogue = EPI_STORE_F64;
    if ((e = launch_gemm64_nt(g, true, true, st)) != hipSuccess) return e;
    for (int J = 0; J < nblk; ++J) {
      const int below = P - (J + 1) * NB;
      const int wgs = below > 0 ? (below + 255) / 256 : 1;
      hipLaunchKernelGGL(chol_step_kernel, dim3((unsigned)(B * wgs)), dim3(256), 0, st, S, D, P, J, wgs, (const int*)nullptr);
      if (below > 0) {
        GemmArgs u;   // trailing block -= panel panel^T
        u.A = S + (long)(J + 1) * NB * P + (long)J * NB; u.B = u.A; u.C = S + (long)(J + 1) * NB * P + (long)(J + 1) * NB;
        u.M = below; u.N = below; u.K = NB; u.lda = P; u.ldb = P; u.ldc = P;
        u.batch = B; u.strideA = (long)P * P; u.strideB = (long)P * P; u.strideC = (long)P * P;
        u.epilogue = EPI_SUB_F64;
        if ((e = launch_gemm64_nt(u, true, true, st)) != hipSuccess) return e;
      }
    }
    const int cw = (nP + 255) / 256;
    for (int bi = 0; bi < nblk; ++bi) {
      if (bi > 0) {
        GemmArgs u;   // X[bi] -= L[bi, 0:bi] X[0:bi]
        u.A = S + (long)bi * NB * P; u.B = X; u.C = X + (long)bi * NB * nP;
        u.M = NB; u.N = nP; u.K = bi * NB; u.lda = P; u.ldb = nP; u.ldc = nP; u.transB = true;
        u.batch = B; u.strideA = (long)P * P; u.strideB = (long)P * nP; u.strideC = (long)P * nP;
        u.epilogue = EPI_SUB_F64;
        if ((e = launch_gemm64_nt(u, true, true, st)) != hipSuccess) return e;
      }
      hipLaunchKernelGGL(solve64_kernel, dim3((unsigned)(B * cw)), dim3(256), 0, st, X, D, P, nP, bi, cw, (const int*)nullptr);
    }
    return hipGetLastError();
  };

  // start block: Omega G
  hipLaunchKernelGGL(omega_kernel, dim3((unsigned)(((long)P * nP + 255) / 256)), dim3(256), 0, st, Om, P, n, nP);
  if (probe_begin && (e = hipEventRecord(probe_begin, st)) != hipSuccess) return e;
  {
    GemmArgs g;
    g.A = Om; g.B = G; g.C = Yt; g.M = P; g.N = nP; g.K = nP; g.lda = nP; g.ldb = nP; g.ldc = nP;
    g.batch = B; g.strideA = 0; g.strideB = (long)nP * nP; g.strideC = (long)P * nP;
    g.epilogue = EPI_STORE_F64;
    if ((e = launch_gemm64_nt(g, true, true, st)) != hipSuccess) return e;
  }
  if (probe_end && (e = hipEventRecord(probe_end, st)) != hipSuccess) return e;
  double* cur = Yt;
  double* oth = Zt;
  for (int it = 0; it < iters; ++it) {
    if ((e = cholqr(cur)) != hipSuccess) return e;
    if (it + 1 == iters && (e = cholqr(cur)) != hipSuccess) return e;   // second pass: orthonormal to rounding
    if ((e = gemm_yt_g(cur, oth)) != hipSuccess) return e;               // oth = Q^T G
    double* t = cur; cur = oth; oth = t;
  }
  // now oth = Q^T (orthonormal rows), cur = Q^T G.  Rayleigh-Ritz: H = (Q^T G) Q
  {
    GemmArgs g;
    g.A = cur; g.B = oth; g.C = H; g.M = P; g.N = P; g.K = nP; g.lda = nP; g.ldb = nP; g.ldc = P;
    g.batch = B; g.strideA = (long)P * nP; g.strideB = (long)P * nP; g.strideC = (long)P * P;
    g.epilogue = EPI_STORE_F64;
    if ((e = launch_gemm64_nt(g, true, true, st)) != hipSuccess) return e;
  }
  if ((e = launch_jacobi_eigen(H, B, P, P, r, jacobi_ctl, jacobi_len2, nullptr, st)) != hipSuccess) return e;
  // rows of H are now theta_k w_k^T; Ut = H Q^T has rows theta_k u_k^T
  {
    GemmArgs g;
    g.A = H; g.B = oth; g.C = cur; g.M = P; g.N = nP; g.K = P; g.lda = P; g.ldb = nP; g.ldc = nP; g.transB = true;
    g.batch = B; g.strideA = (long)P * P; g.strideB = (long)P * nP; g.strideC = (long)P * nP;
    g.epilogue = EPI_STORE_F64;
    if ((e = launch_gemm64_nt(g, true, true, st)) != hipSuccess) return e;
  }
  // residuals: Rt = Ut G
  if ((e = gemm_yt_g(cur, oth)) != hipSuccess) return e;
  if ((e = launch_row_lengths(cur, B, P, nP, (long)P * nP, lam, st)) != hipSuccess) return e;
  hipLaunchKernelGGL(ritz_check_kernel, dim3(B), dim3(256), 0, st, cur, oth, lam, P, n, nP, r, 1e-10, ok);
  *ut = cur;
  return hipGetLastError();
}

}  // namespace covspec
