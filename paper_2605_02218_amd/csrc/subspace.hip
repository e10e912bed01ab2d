// Top-r eigen-subspace of the token Gram matrix by block subspace iteration
// (the rank-r truncated SVD of paper Sec. III-A.3 only needs V_r and Sigma_r).
//
// Only the r dominant eigenpairs of G = Z_M^T Z_M enter the energies, so instead of
// diagonalising all of G, a block of P > r vectors is iterated:
//     Y <- G Y,  Y <- orthonormalise(Y)          (P = r + 64..127; error shrinks by lambda_{P+1}/lambda_r per step)
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
#include "host_cache.h"
#include "kernels.h"

namespace covspec {

namespace {

constexpr int NB = 64;        // panel width of Cholesky / substitution
constexpr int NBP = NB + 1;   // LDS pitch
// Relative residual |G u - theta u| / theta accepted for the r dominant Ritz pairs.  The Jacobi solve of the
// projected problem stops at an admixture weight that leaves the energies good to ~1e-8, and a residual of
// 1e-9 perturbs an energy by at most 1e-9 / (relative gap at r) relative, the same order; converged blocks
// sit at 1e-11..1e-13, unconverged ones orders above.
constexpr double kRitzTol = 1e-9;
// see the end of chol_kernel
constexpr double kPivotNear = 0.25;   // smallest scaled pivot above this: rows nearly orthogonal, blocks of three steps
constexpr double kPivotFar = 1e-3;    // above this: blocks of two steps
constexpr double kGradeDigits = 14.0; // decimal digits a block's grading (lambda_1 / lambda_P)^steps may use up
constexpr int kMaxBlockSteps = 3;
// Couplings between rows of the projected matrix below this weight are left out of the first, banded sweeps of the
// Ritz solve (its last sweeps visit every pair).
constexpr double kBandTol = 1e-9;
constexpr double kPivotOnePass = 0.01; // final step: above this one Cholesky-QR pass leaves the rows orthonormal to ~1e-14
constexpr size_t kCholLdsFixed = (size_t)(2 * NB * NBP + NB) * sizeof(double);   // plus P doubles: the diagonal of S

__global__ void omega_kernel(double* __restrict__ om, int P, int n, int nP) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long)P * nP) return;
  const int r = (int)(i / nP), c = (int)(i - (long)r * nP);
  uint32_t h = (uint32_t)r * 0x9E3779B1u ^ ((uint32_t)c + 0x7F4A7C15u) * 0x85EBCA77u;
  h ^= h >> 15; h *= 0x2C1B3C6Du; h ^= h >> 12; h *= 0x297A2D39u; h ^= h >> 15;
  om[i] = (c < n) ? ((h & 1u) ? 1.0 : -1.0) : 0.0;
}

// value of `v` in lane `l` (compile-time lane), uniform across the wave
template <typename = void>
__device__ __forceinline__ double lane_value(double v, int l) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), l), hi = __builtin_amdgcn_readlane(__double2hiint(v), l);
  return __hiloint2double(hi, lo);
}

// Factors the 64 x 64 block `a` (LDS, pitch NBP, lower triangle) in one wave: lane i holds row i.  The factor
// goes to `fac` (lower triangle, zeros above).  Pivots are floored at `floor_`.  Column k: pivot from lane k, scaled
// column l_ik = a_ik / sqrt(a_kk) (lane i), then a_ij -= l_ik l_jk.  The l_jk of the other lanes come through
// `col` (64 doubles of LDS): every lane posts its l_ik and reads the column back as broadcast loads, two values
// per load (a wave's LDS accesses complete in order, so no barrier is needed; reading them lane by lane with
// v_readlane took two such instructions and their wait states per value and ran at twice the time).  Not inlined,
// so that the 64 row registers do not compete with the caller's.
__device__ __noinline__ void potrf_wave(const double* a, double* fac, double* col, double floor_) {
  const int lane = threadIdx.x & 63;
  double row[NB];
#pragma unroll
  for (int k = 0; k < NB; ++k) row[k] = a[lane * NBP + k];
#pragma unroll
  for (int k = 0; k < NB; ++k) {
    const double akk = fmax(lane_value(row[k], k), floor_);
    double rs = __builtin_amdgcn_rsq(akk);
    rs = rs * fma(-0.5 * akk, rs * rs, 1.5);
    rs = rs * fma(-0.5 * akk, rs * rs, 1.5);
    const double lk = (lane == k) ? akk * rs : row[k] * rs;
    row[k] = lk;
    if (k + 1 < NB) {
      col[lane] = lk;
#pragma unroll
      for (int j = k + 1; j < NB; ++j) row[j] = fma(-lk, col[j], row[j]);
    }
  }
#pragma unroll
  for (int k = 0; k < NB; ++k) fac[lane * NBP + k] = (k <= lane) ? row[k] : 0.0;
}

// Cholesky factorisation S[b] = L L^T (P x P, pitch P, P % 64 == 0; only the lower triangle is read), one
// 512-thread workgroup per image, right-looking over 64-wide panels:
//   diagonal block: factored in LDS, then inverted in LDS; the inverse goes to Dinv[b][J] (64 x 64);
//   panel below:    X = S[I,J] inv(L_JJ)^T on the MFMA, in place (these blocks are L[I,J]);
//   trailing part:  S[I,I'] -= X_I X_I'^T for I' <= I on the MFMA, 16 x 64 units dealt round-robin to the waves.
// On return the strictly-lower blocks of S hold L; its diagonal blocks are represented by their inverses.
// Pivots are floored at 1e-28 * trace(first block) so that a numerically rank-deficient block cannot
// produce NaNs (the residual check afterwards decides whether the result is usable).
// Dynamic LDS: 2 * 64 * 65 + 64 + P doubles.
__global__ __launch_bounds__(512) void chol_kernel(double* S, double* __restrict__ Dinv, int P, int* skip_until, int* last_orth, int step,
                                                   int last_free_step, int next_weight) {
  extern __shared__ double lds[];
  double* a = lds;                  // [64][65] diagonal block, later the inverse of its factor
  double* fac = lds + NB * NBP;     // [64][65] the factor (lower triangle) and scratch (upper triangle)
  double* col = lds + 2 * NB * NBP;     // [64] column exchange of the one-wave factorisation
  double* diag0 = col + NB;             // [P] the diagonal of S before any update: squared row lengths
  const int b = blockIdx.x;
  if (skip_until && skip_until[b] > step) return;   // this image does not orthonormalise at this step
  double* Sb = S + (long)b * P * P;
  double dmin = 1e300, dmax = 0.0, pmin = 1.0;   // extremes of the factor's diagonal, smallest scaled pivot (thread 0)
  const int nblk = P / NB;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, i16 = lane & 15, kq = lane >> 4;
  double floor_ = 0.0;
  for (int k = tid; k < P; k += 512) diag0[k] = Sb[(long)k * P + k];

  // The diagonal block of the first panel: factored by ONE wave, row i of the block in the registers of lane i (no
  // barrier and no LDS traffic per column; with the whole workgroup a column cost a barrier and a round trip through
  // LDS, and the factorisation is a chain of 64 dependent columns).  Column k: pivot from lane k, scaled column
  // l_ik = a_ik / sqrt(a_kk), then a_ij -= l_ik l_jk with l_jk read from lane j.  Lanes also carry the (unused)
  // entries above the diagonal; they stay finite and never feed an entry below it.
  for (int e = tid; e < NB * NB; e += 512) {
    const int i = e >> 6, j = e & 63;
    a[i * NBP + j] = (j <= i) ? Sb[(long)i * P + j] : 0.0;
  }
  __syncthreads();
  {
    double tr = 0.0;
    for (int i = 0; i < NB; ++i) tr += a[i * NBP + i];   // same value in every thread
    floor_ = 1e-300 + 1e-28 * tr;
  }
  if (w == 0) potrf_wave(a, fac, col, floor_);
  __syncthreads();

  for (int J = 0; J < nblk; ++J) {
    const int j0 = J * NB;
    // here `fac` holds the factor of diagonal block J (for J > 0 wave 0 formed it during the trailing update of panel J - 1)
    if (tid == 0)
      for (int k = 0; k < NB; ++k) {
        const double d = fac[k * NBP + k];
        dmin = fmin(dmin, d);
        dmax = fmax(dmax, d);
        const double s0 = diag0[j0 + k];
        if (s0 > 0.0) pmin = fmin(pmin, d * d / s0);
      }
    // ---- inverse of the factor into `a`, by doubling: with L = [A 0; C D], inv(L) = [inv(A) 0; -inv(D) C inv(A) inv(D)].
    //      Level s joins the inverses of the s x s diagonal blocks pairwise; the intermediate C inv(A) is parked,
    //      transposed, in the unused upper triangle of `fac`.
    for (int e = tid; e < NB * NB; e += 512) {
      const int i = e >> 6, j = e & 63;
      a[i * NBP + j] = (i == j) ? 1.0 / fac[i * NBP + i] : 0.0;
    }
    __syncthreads();
    for (int s_ = 1, ls = 0; s_ < NB; s_ <<= 1, ++ls) {
      // 32 * s_ elements per level: element e -> block pair m, row i, column j
      for (int e = tid; e < 32 * s_; e += 512) {
        const int m = e >> (2 * ls), i = (e >> ls) & (s_ - 1), j = e & (s_ - 1);
        const int base = 2 * s_ * m;
        double t1 = 0.0;   // (C inv(A))[i][j], inv(A) lower triangular
#pragma unroll 8
        for (int t = j; t < s_; ++t) t1 = fma(fac[(base + s_ + i) * NBP + base + t], a[(base + t) * NBP + base + j], t1);
        fac[(base + j) * NBP + base + s_ + i] = t1;
      }
      __syncthreads();
      for (int e = tid; e < 32 * s_; e += 512) {
        const int m = e >> (2 * ls), i = (e >> ls) & (s_ - 1), j = e & (s_ - 1);
        const int base = 2 * s_ * m;
        double x = 0.0;    // (inv(D) T1)[i][j], inv(D) lower triangular
#pragma unroll 8
        for (int u = 0; u <= i; ++u) x = fma(a[(base + s_ + i) * NBP + base + s_ + u], fac[(base + j) * NBP + base + s_ + u], x);
        a[(base + s_ + i) * NBP + base + j] = -x;
      }
      __syncthreads();
    }
    double* inv = a;
    {
      double* Db = Dinv + ((long)b * nblk + J) * NB * NB;
      // stored with the columns of every group of 16 permuted, 16x + 4v + q -> 16x + 4q + v: trsm_kernel's lane
      // of quarter q contracts the columns 16x + 4v + q, v = 0..3, of a step group and reads them as one 32-byte piece
      for (int e = tid; e < NB * NB; e += 512) {
        const int c = e & 63;
        Db[(e & ~63) | (c & 48) | ((c & 3) << 2) | ((c >> 2) & 3)] = inv[(e >> 6) * NBP + c];
      }
    }
    // ---- panel: X = S[I,J] inv^T, 16-row tiles dealt to the waves
    const int below = P - j0 - NB;
    for (int t = w; t < below / 16; t += 8) {
      const long rb = j0 + NB + 16 * t;
      f64x4_t f[4], out[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) f[c] = *(const f64x4_t*)(Sb + (rb + i16) * P + j0 + 16 * c + 4 * kq);
#pragma unroll
      for (int y = 0; y < 4; ++y) {
        out[y] = (f64x4_t){0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
          for (int jj = 0; jj < 4; ++jj)
            out[y] = __builtin_amdgcn_mfma_f64_16x16x4f64(f[c][jj], inv[(16 * y + i16) * NBP + 16 * c + 4 * kq + jj], out[y], 0, 0, 0);
      }
#pragma unroll
      for (int y = 0; y < 4; ++y)
#pragma unroll
        for (int v = 0; v < 4; ++v) Sb[(rb + 4 * v + kq) * P + j0 + 16 * y + i16] = out[y][v];
    }
    __syncthreads();     // the panel is complete in global memory and `a`, `fac` are free
    if (below == 0) break;
    // ---- trailing update, unit = 16 rows of block I x the 64 columns of block I' <= I.  The four units of the
    //      next diagonal block go to wave 0, which writes them to LDS instead of global memory and factors the
    //      block at once (look-ahead: the chain of 64 dependent columns runs beside the rest of the update instead
    //      of after it); the other waves share the remaining units in contiguous ranges, so that consecutive units
    //      mostly share I' and its fragments stay in registers.  All loads of a unit are issued before its MFMAs.
    {
      const int nb = below / NB;
      const int units = 2 * nb * (nb + 1);            // 4 * nb (nb + 1) / 2; units 0..3 are the next diagonal block
      int u0, u1;
      if (w == 0) { u0 = 0; u1 = 4; }
      else { u0 = 4 + (int)((long)(units - 4) * (w - 1) / 7); u1 = 4 + (int)((long)(units - 4) * w / 7); }
      // unit u -> pair index u / 4 -> (I, I2) with I (I + 1) / 2 + I2 = pair index
      int I = 0, I2 = 0;
      {
        int pi = u0 >> 2;
        while ((I + 1) * (I + 2) / 2 <= pi) ++I;
        I2 = pi - I * (I + 1) / 2;
      }
      f64x4_t fb[4][4];
      int have = -1;
      for (int u = u0; u < u1; ++u) {
        const int q = u & 3;
        const long ra = j0 + NB + (long)I * NB + 16 * q;
        const long rc = j0 + NB + (long)I2 * NB;
        f64x4_t fa[4], cc[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) fa[c] = *(const f64x4_t*)(Sb + (ra + i16) * P + j0 + 16 * c + 4 * kq);
        if (have != I2) {
#pragma unroll
          for (int y = 0; y < 4; ++y)
#pragma unroll
            for (int c = 0; c < 4; ++c) fb[y][c] = *(const f64x4_t*)(Sb + (rc + 16 * y + i16) * P + j0 + 16 * c + 4 * kq);
          have = I2;
        }
        f64x4_t acc[4];
#pragma unroll
        for (int y = 0; y < 4; ++y) acc[y] = (f64x4_t){0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
          for (int y = 0; y < 4; ++y)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) acc[y] = __builtin_amdgcn_mfma_f64_16x16x4f64(fa[c][jj], fb[y][c][jj], acc[y], 0, 0, 0);
#pragma unroll
        for (int y = 0; y < 4; ++y)
#pragma unroll
          for (int v = 0; v < 4; ++v) cc[y][v] = Sb[(ra + 4 * v + kq) * P + rc + 16 * y + i16];
        if (w == 0) {
          // the next diagonal block (every entry of it is kept up to date, above the diagonal too): into LDS
#pragma unroll
          for (int y = 0; y < 4; ++y)
#pragma unroll
            for (int v = 0; v < 4; ++v) a[(16 * q + 4 * v + kq) * NBP + 16 * y + i16] = cc[y][v] - acc[y][v];
        } else {
#pragma unroll
          for (int y = 0; y < 4; ++y)
#pragma unroll
            for (int v = 0; v < 4; ++v) Sb[(ra + 4 * v + kq) * P + rc + 16 * y + i16] = cc[y][v] - acc[y][v];
        }
        if (q == 3) {   // next pair
          if (I2 == I) { ++I; I2 = 0; } else ++I2;
        }
      }
      if (w == 0) {
        // one wave wrote the block and one wave reads it: its LDS writes are complete once the counter says so
        __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
        __builtin_amdgcn_wave_barrier();
        potrf_wave(a, fac, col, floor_);
      }
    }
    __syncthreads();
  }
  // How many steps (products with G) the image may take before it orthonormalises again.  Two things limit a
  // block of m steps.  (1) Cholesky-QR needs the SCALED Gram matrix (unit diagonal) to be well conditioned; the raw
  // grading lambda_1 / lambda_P of the rows is harmless.  The scaled pivots L_kk^2 / S_kk (squared sine of the
  // angle between row k and the rows before it) say how close to orthogonal the rows were: the iteration orders
  // the rows like the eigenvectors, and once it has, they stay nearly orthogonal over several steps.  (2) Within a
  // row the wanted direction must not drown in rounding noise along the dominant one: (lambda_1 / lambda_P)^m has
  // to stay well inside the 16 digits; the diagonal of L spans that ratio for the steps of the block just closed.
  if (tid == 0 && skip_until) {
    int m = 1;
    if (step >= 1 && dmin > 0.0) {
      const int closed = step - last_orth[b];                       // steps in the block just factored (>= 1)
      const double digits_per_step = log10(fmax(dmax / dmin, 10.0)) / (double)(closed < 1 ? 1 : closed);
      const int by_grade = (int)(kGradeDigits / digits_per_step);
      const int by_pivot = pmin > kPivotNear ? kMaxBlockSteps : (pmin > kPivotFar ? 2 : 1);
      // by_pivot counts products with G; the products that follow multiply by G^next_weight.  by_grade is in
      // products of the block just closed, whose weight is never below that of the next ones.
      const int by_pivot_products = by_pivot / next_weight;
      m = by_pivot_products < by_grade ? by_pivot_products : by_grade;
      if (m < 1) m = 1;
    }
    int next = step + m;                      // the next step that orthonormalises
    if (next > last_free_step) next = last_free_step;     // the final step always does
    // The final step is followed by a second pass (step + 1) that makes the rows orthonormal to rounding; the
    // error of one pass is about 1e-16 times the scaled condition number, so with large pivots it is not needed.
    if (step == last_free_step) next = pmin > kPivotOnePass ? step + 2 : step + 1;
    skip_until[b] = next;
    last_orth[b] = step;
  }
}

// Yt[b] <- L^-1 Yt[b] (P x nP, pitch nP) by blocked forward substitution with the factor chol_kernel left
// in S (strictly-lower blocks) and Dinv (inverted diagonal blocks).  Columns are independent: each wave
// owns 16 of them and never reads what another wave writes, so the whole solve is one launch.
//   for block row bi:  T = Yt[bi] - sum_{K<bi} L[bi,K] Yt[K];   Yt[bi] = inv(L_bibi) T
// T comes out of the MFMA in exactly the layout its B operand wants (lane = column, register = k), so the
// second product takes the accumulator registers as they are.
__global__ __launch_bounds__(256) void trsm_kernel(double* Yt, const double* __restrict__ S, const double* __restrict__ Dinv,
                                                    int P, int nP, int wg_per_image, const int* __restrict__ last_orth, int step) {
  const int b = blockIdx.x / wg_per_image, cw = blockIdx.x - b * wg_per_image;
  if (last_orth && last_orth[b] != step) return;    // the factorisation of this step did not run for this image
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, i16 = lane & 15, kq = lane >> 4;
  const int col = cw * 64 + w * 16 + i16;    // nP % 64 == 0, so every column exists
  const int nblk = P / NB;
  double* Yb = Yt + (long)b * P * nP;
  const double* Lb = S + (long)b * P * P;
  for (int bi = 0; bi < nblk; ++bi) {
    f64x4_t acc[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) acc[x] = (f64x4_t){0.0, 0.0, 0.0, 0.0};
    for (int kk = 0; kk < bi * NB; kk += 16) {
      f64x4_t fa[4];
      double fb[4];
#pragma unroll
      for (int x = 0; x < 4; ++x) fa[x] = *(const f64x4_t*)(Lb + (long)(bi * NB + 16 * x + i16) * P + kk + 4 * kq);
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) fb[jj] = Yb[(long)(kk + 4 * kq + jj) * nP + col];
#pragma unroll
      for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) acc[x] = __builtin_amdgcn_mfma_f64_16x16x4f64(fa[x][jj], fb[jj], acc[x], 0, 0, 0);
    }
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[x][v] = Yb[(long)(bi * NB + 16 * x + 4 * v + kq) * nP + col] - acc[x][v];
    const double* Db = Dinv + ((long)b * nblk + bi) * NB * NB;
    f64x4_t out[4];
#pragma unroll
    for (int a = 0; a < 4; ++a) out[a] = (f64x4_t){0.0, 0.0, 0.0, 0.0};
    // step (x, v) contracts k = 16x + 4v + kq, the row acc[x][v] holds in this lane; the inverse block is stored
    // with its columns permuted so that the four v of a group are contiguous.  Two groups of loads in flight.
#pragma unroll
    for (int xh = 0; xh < 4; xh += 2) {
      f64x4_t da[2][4];
#pragma unroll
      for (int xx = 0; xx < 2; ++xx)
#pragma unroll
        for (int a = 0; a < 4; ++a) da[xx][a] = *(const f64x4_t*)(Db + (16 * a + i16) * NB + 16 * (xh + xx) + 4 * kq);
#pragma unroll
      for (int xx = 0; xx < 2; ++xx)
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
          for (int a = 0; a < 4; ++a) out[a] = __builtin_amdgcn_mfma_f64_16x16x4f64(da[xx][a][v], acc[xh + xx][v], out[a], 0, 0, 0);
    }
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int v = 0; v < 4; ++v) Yb[(long)(bi * NB + 16 * a + 4 * v + kq) * nP + col] = out[a][v];
    __threadfence_block();   // the rows just written are B operands of the next block rows
  }
}

// skip_until[b] = ok[b] ? INT_MAX : -1 (images that passed take no further part), last_orth[b] = -1
__global__ void mask_passed_kernel(const int* __restrict__ ok, int* __restrict__ skip_until, int* __restrict__ last_orth, int B) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  skip_until[b] = ok[b] ? 0x7fffffff : -1;
  last_orth[b] = -1;
}

// Residual check of the r dominant Ritz pairs.  Ut rows are theta_k u_k^T, Rt = Ut G.  ok[b] = 1 (2 in the second pass) when
// |Rt_k - theta_k Ut_k| <= tol * theta_k^2 for each of them (theta_k = |Ut_k|, so this is the relative
// residual |G u - theta u| / theta).
__global__ __launch_bounds__(1024) void ritz_check_kernel(const double* __restrict__ Ut, const double* __restrict__ Rt,
                                                           const double* __restrict__ lam, int P, int n, int nP, int r,
                                                           double tol, int* ok, int only_failed) {
  __shared__ double slam[4096];
  __shared__ unsigned char sel[4096];
  __shared__ int bad;
  const int b = blockIdx.x, lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  if (only_failed && ok[b]) return;      // passed an earlier check; its rows were not touched since (uniform)
  const double* lb = lam + (long)b * P;
  for (int k = threadIdx.x; k < P; k += 1024) slam[k] = lb[k];
  if (threadIdx.x == 0) bad = 0;
  __syncthreads();
  for (int k = threadIdx.x; k < P; k += 1024) {
    const double v = slam[k];
    int rank = 0;
    for (int j = 0; j < P; ++j) { const double u = slam[j]; rank += (u > v || (u == v && j < k)) ? 1 : 0; }
    sel[k] = rank < r;
  }
  __syncthreads();
  // one wave per row, four pairs of loads in flight per lane
  for (int k = w; k < P; k += 16) {
    if (!sel[k]) continue;
    const double th = slam[k];
    const double* u = Ut + ((long)b * P + k) * nP;
    const double* rr = Rt + ((long)b * P + k) * nP;
    double s0 = 0.0, s1 = 0.0;
    int j = lane;
    for (; j + 192 < n; j += 256) {
      double a[4], c[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) { a[q] = rr[j + 64 * q]; c[q] = u[j + 64 * q]; }
#pragma unroll
      for (int q = 0; q < 4; q += 2) {
        const double d0 = a[q] - th * c[q], d1 = a[q + 1] - th * c[q + 1];
        s0 = fma(d0, d0, s0);
        s1 = fma(d1, d1, s1);
      }
    }
    for (; j < n; j += 64) { const double d = rr[j] - th * u[j]; s0 = fma(d, d, s0); }
    const double s = wave_sum(s0 + s1);
    if (lane == 0 && !(sqrt(s) <= tol * th * th)) bad = 1;   // also catches NaN
  }
  __syncthreads();
  if (threadIdx.x == 0) ok[b] = bad ? 0 : (only_failed ? 2 : 1);    // 1: first pass, 2: second pass
}

}  // namespace

int subspace_block(int n, int r) {
  // P = r + 64 rounded up to the panel width: the Ritz problem costs P^3 and each step P^2 n, while a wider
  // block only buys a better contraction factor lambda_{P+1}/lambda_r per step, so the narrow block with a
  // few more steps is the cheaper trade.  0 = not worthwhile (P would be most of n).
  int P = (r + 64 + NB - 1) / NB * NB;
  return (4 * P <= 3 * n) ? P : 0;
}

size_t subspace_workspace_bytes(int B, int n, int nP, int P) {
  if (P <= 0) return 0;
  const size_t blk = (size_t)B * P * nP * 8;
  return 2 * blk + (size_t)P * nP * 8 + 2 * (size_t)B * P * P * 8 + (size_t)B * P * NB * 8 + (size_t)B * P * 8 + 1024 + (size_t)B * 4 +
         (size_t)B * 4 + (size_t)B * 4 /* band limits */ + 256 + (size_t)B * nP * nP * 8 /* G^2 */ + 256;
}

// Runs the iteration on G[b] (n x n, pitch nP, untouched).  On return, for images with ok[b] = 1, rows
// k of (*ut)[b] (P rows, pitch nP, inside ws) are theta_k u_k^T with the r longest rows converged.
// The first pass makes iters steps of the iteration as iters / 3 products with G^2 followed by iters / 3 with G.
// Launches of the probed shape: start block, the products of the first pass, residuals.
int subspace_product_launches(int iters) { return 2 * (iters / 3) + 2; }

hipError_t launch_subspace_eigen(const double* G, int B, int n, int nP, int r, int P, int iters, int more_iters, void* ws_, void* jacobi_ctl,
                                 double* jacobi_len2, int* ok, const double** ut, int* img_status, hipEvent_t probe_begin,
                                 hipEvent_t probe_end, hipStream_t st) {
  hipError_t e0;
  if (P <= 0 || P % NB != 0 || P > n || P > 4096 || nP % NB != 0) return hipErrorInvalidValue;
  // every pass makes an even number of products, so that the rows of the images that passed the first check are
  // in the block that is returned (the two blocks swap roles per product)
  if (iters < 3 || iters % 3 != 0 || more_iters < 2 || (more_iters & 1)) return hipErrorInvalidValue;
  {
    static PerDeviceInt raised;
    if ((e0 = ensure_dynamic_lds(raised, (const void*)chol_kernel, kCholLdsFixed + 4096 * sizeof(double))) != hipSuccess) return e0;
  }
  char* ws = (char*)ws_;
  const size_t blk = (size_t)B * P * nP * 8;
  double* Yt = (double*)ws;                 // after the call: Ut
  double* Zt = (double*)(ws + blk);
  double* Om = (double*)(ws + 2 * blk);
  double* S = (double*)(ws + 2 * blk + (size_t)P * nP * 8);
  double* H = S + (size_t)B * P * P;
  double* D = H + (size_t)B * P * P;
  double* lam = D + (size_t)B * P * NB;
  int* skip_until = (int*)(((uintptr_t)(lam + (size_t)B * P) + 255) & ~(uintptr_t)255);   // [B] next step that orthonormalises
  int* last_orth = skip_until + B;                                                          // [B] step of the last one
  int* band = last_orth + B;                                                                // [B] see launch_band_limit
  double* G2 = (double*)(((uintptr_t)(band + B) + 255) & ~(uintptr_t)255);                  // [B][nP][nP] G squared
  const int nblk = P / NB;
  hipError_t e;

  // Second pass: images that passed the first check take no further part; the kernels see them as skip_until ==
  // INT_MAX (never reached by a step counter), which is what `masked` switches on for the plain products.
  bool masked = false;
  auto mask = [&](GemmArgs& g) {
    if (masked) { g.skip = skip_until; g.skip_if = 0x7ffffffe; }
  };
  auto gemm_yt_g = [&](const double* X, double* out, const double* Gop) {   // out = X Gop  (P x nP), Gop = G or G^2
    GemmArgs g;
    g.A = X; g.B = Gop; g.C = out; g.M = P; g.N = nP; g.K = nP; g.lda = nP; g.ldb = nP; g.ldc = nP;
    g.batch = B; g.strideA = (long)P * nP; g.strideB = (long)nP * nP; g.strideC = (long)P * nP;
    g.epilogue = EPI_STORE_F64;
    mask(g);
    return launch_gemm64_nt(g, true, true, st);
  };
  // X <- L^-1 X with X X^T = L L^T.  Images with skip_until[b] > step leave X alone, and the factorisation decides
  // how many steps the image takes before the next one (never beyond last_free_step).
  const size_t chol_lds = kCholLdsFixed + (size_t)P * sizeof(double);
  auto cholqr = [&](double* X, int step, int last_free_step, int next_weight) -> hipError_t {
    GemmArgs g;
    g.A = X; g.B = X; g.C = S; g.M = P; g.N = P; g.K = nP; g.lda = nP; g.ldb = nP; g.ldc = P;
    g.batch = B; g.strideA = (long)P * nP; g.strideB = (long)P * nP; g.strideC = (long)P * P;
    g.epilogue = EPI_STORE_F64;
    g.lower_only = true;
    g.skip = skip_until;
    g.skip_if = step;
    if ((e = launch_gemm64_nt(g, true, true, st)) != hipSuccess) return e;
    hipLaunchKernelGGL(chol_kernel, dim3((unsigned)B), dim3(512), chol_lds, st, S, D, P, skip_until, last_orth, step, last_free_step,
                       next_weight);
    hipLaunchKernelGGL(trsm_kernel, dim3((unsigned)(B * (nP / NB))), dim3(256), 0, st, X, (const double*)S, (const double*)D, P, nP,
                       nP / NB, (const int*)last_orth, step);
    return hipGetLastError();
  };
  double* cur = Yt;
  double* oth = Zt;
  // `steps` products from the block in `cur` (each preceded by an orthonormalisation where the image's schedule
  // asks for one), then Rayleigh-Ritz and the residual check.  steps is even, so `cur` is the same buffer after it.
  // The first n_sq products multiply by G^2: two steps of the iteration at the cost of one (the same subspace as
  // two products with G and an orthonormalisation between them).  G^2 as formed is off by about 1e-16 |G|^2, which
  // is a fixed perturbation of the operator of relative size 1e-16 (lambda_1 / lambda_r)^2 at the r-th eigenvalue
  // (1e-8 for a spectrum that falls by 1e4 down to r); the products with G itself that follow contract that error
  // like any other, and a CPU model of the workloads' matrices needs three to four of them.  The last product
  // feeds the Rayleigh-Ritz step and is with G in any case.
  auto pass = [&](int n_sq, int n_plain) -> hipError_t {
    const int steps = n_sq + n_plain;
    for (int it = 0; it < steps; ++it) {
      // the block of step 0 is not (orthonormal) x G, so its factor says nothing about the next step (the kernel
      // takes one step after it); the last step always orthonormalises, twice where its pivots ask for it
      const int w = it < n_sq ? 2 : 1;
      if ((e = cholqr(cur, it, steps - 1, w)) != hipSuccess) return e;
      if (it + 1 == steps && (e = cholqr(cur, it + 1, steps - 1, 1)) != hipSuccess) return e;
      if ((e = gemm_yt_g(cur, oth, w == 2 ? G2 : G)) != hipSuccess) return e;   // last: oth = Q^T G
      double* t = cur; cur = oth; oth = t;
    }
    // now oth = Q^T (orthonormal rows), cur = Q^T G.  Rayleigh-Ritz: H = (Q^T G) Q
    {
      GemmArgs g;
      g.A = cur; g.B = oth; g.C = H; g.M = P; g.N = P; g.K = nP; g.lda = nP; g.ldb = nP; g.ldc = P;
      g.batch = B; g.strideA = (long)P * nP; g.strideB = (long)P * nP; g.strideC = (long)P * P;
      g.epilogue = EPI_STORE_F64;
      g.lower_only = true;      // H is symmetric: the tiles below the diagonal are mirrored
      g.mirror = true;
      mask(g);
      if ((e = launch_gemm64_nt(g, true, true, st)) != hipSuccess) return e;
    }
    // The rows of the block are ordered like the eigenvalues, so H only couples neighbouring rows: measure how far
    // (on H^2, the Gram matrix of the rows the solve rotates; S is free by now) and let the solve leave the rest out
    {
      GemmArgs g;
      g.A = H; g.B = H; g.C = S; g.M = P; g.N = P; g.K = P; g.lda = P; g.ldb = P; g.ldc = P;
      g.batch = B; g.strideA = (long)P * P; g.strideB = (long)P * P; g.strideC = (long)P * P;
      g.epilogue = EPI_STORE_F64;
      g.lower_only = true;
      mask(g);
      if ((e = launch_gemm64_nt(g, true, true, st)) != hipSuccess) return e;
      if ((e = launch_band_limit(S, B, P, kBandTol, band, masked ? (const int*)ok : nullptr, st)) != hipSuccess) return e;
    }
    if ((e = launch_jacobi_eigen(H, B, P, P, r, jacobi_ctl, jacobi_len2, masked ? (const int*)ok : nullptr, band, img_status, st)) != hipSuccess) return e;
    // rows of H are now theta_k w_k^T; Ut = H Q^T has rows theta_k u_k^T
    {
      GemmArgs g;
      g.A = H; g.B = oth; g.C = cur; g.M = P; g.N = nP; g.K = P; g.lda = P; g.ldb = nP; g.ldc = nP; g.transB = true;
      g.batch = B; g.strideA = (long)P * P; g.strideB = (long)P * nP; g.strideC = (long)P * nP;
      g.epilogue = EPI_STORE_F64;
      mask(g);
      if ((e = launch_gemm64_nt(g, true, true, st)) != hipSuccess) return e;
    }
    // residuals: Rt = Ut G
    if ((e = gemm_yt_g(cur, oth, G)) != hipSuccess) return e;
    if ((e = launch_row_lengths(cur, B, P, nP, (long)P * nP, lam, st)) != hipSuccess) return e;
    hipLaunchKernelGGL(ritz_check_kernel, dim3(B), dim3(1024), 0, st, cur, oth, lam, P, n, nP, r, kRitzTol, ok, masked ? 1 : 0);
    return hipGetLastError();
  };

  // G^2 (symmetric: tiles on and below the diagonal, mirrored)
  {
    GemmArgs g;
    g.A = G; g.B = G; g.C = G2; g.M = nP; g.N = nP; g.K = nP; g.lda = nP; g.ldb = nP; g.ldc = nP;
    g.batch = B; g.strideA = (long)nP * nP; g.strideB = (long)nP * nP; g.strideC = (long)nP * nP;
    g.epilogue = EPI_STORE_F64;
    g.lower_only = true;
    g.mirror = true;
    if ((e = launch_gemm64_nt(g, true, true, st)) != hipSuccess) return e;
  }
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
  if ((e = launch_fill_int(skip_until, 2 * B, -1, st)) != hipSuccess) return e;
  if ((e = pass(iters / 3, iters / 3)) != hipSuccess) return e;
  // images whose Ritz pairs are not there yet (slower spectral decay than the first pass allows for) go on from
  // their Ritz vectors for a few more steps; for the others every kernel of this pass returns at once
  masked = true;
  hipLaunchKernelGGL(mask_passed_kernel, dim3((unsigned)((B + 255) / 256)), dim3(256), 0, st, (const int*)ok, skip_until, last_orth, B);
  if ((e = pass(0, more_iters)) != hipSuccess) return e;
  *ut = cur;
  return hipGetLastError();
}

}  // namespace covspec
