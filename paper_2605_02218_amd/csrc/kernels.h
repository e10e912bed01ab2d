// Host-side launch interface of the gfx950 kernels.  Every launcher enqueues on
// `stream` and returns the launch status; none allocates or synchronises.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace covspec {

enum { DT_F32 = 0, DT_BF16 = 1, DT_F16 = 2 /* logits of the vocabulary passes only */ };

// ---------------------------------------------------------------- gemm.hip
// C[M,N] = A[M,K] * B[N,K]^T  (both operands K-contiguous), fp32 accumulation on MFMA.
enum GemmEpilogue {
  EPI_STORE_F32 = 0,  // C fp32 [M,N]
  EPI_ROWNORM2 = 1,   // C fp32 [M, tiles_n]: per-tile sums over columns of C^2 (C itself is not stored)
  EPI_STORE_F64 = 2,  // C fp64 [M,N]; the fp32 accumulators are flushed into fp64 every 256 k
  EPI_SUB_F64 = 3,    // C fp64 [M,N] -= A*B^T (fp64 kernel only)
};

struct GemmArgs {
  const void* A = nullptr;
  const void* B = nullptr;
  void* C = nullptr;
  int M = 0, N = 0, K = 0;
  long lda = 0, ldb = 0, ldc = 0;              // row pitches, in elements
  int batch = 1;                               // total batch count = outer * batch_inner
  int batch_inner = 1;                         // batch id -> (outer = id / inner, in = id % inner)
  long strideA = 0, strideB = 0, strideC = 0;  // outer batch strides, in elements
  long strideA2 = 0, strideB2 = 0, strideC2 = 0;  // inner batch strides, in elements
  const int32_t* gatherA = nullptr;            // optional [outer batch, M] / [outer batch, N] row lists
  const int32_t* gatherB = nullptr;
  long gstrideA = 0, gstrideB = 0;
  int epilogue = EPI_STORE_F32;
  // fp64 kernel only:
  bool lower_only = false;                     // tiles entirely above the diagonal of C are not computed
  bool mirror = false;                         // with lower_only, square tiles and a symmetric product (A = B): tiles below the
                                               // diagonal are also stored transposed, so that C comes out full
  bool transB = false;                         // B is stored [K][N] (row pitch ldb), i.e. C = A * B
  const int* skip = nullptr;                   // per outer batch: the work is skipped while skip[b] > skip_if
  int skip_if = 1;
};
int gemm_tiles_n(int N);
hipError_t launch_gemm_nt(const GemmArgs& g, int dtype, hipStream_t stream);

// ---------------------------------------------------------------- gemm64.hip
// Same contraction entirely in fp64 (v_mfma_f64_16x16x4); A and B are fp32 or fp64, C is fp64.
// Epilogues: EPI_STORE_F64, EPI_ROWNORM2 (fp64 partials, one per 64-column tile).
int gemm64_tiles_n(int N);
hipError_t launch_gemm64_nt(const GemmArgs& g, bool a_is_f64, bool b_is_f64, hipStream_t stream);
// Both operands bf16: products of bf16 values are exact in fp64 and the sum is fp64, so the result is the
// exactly rounded contraction to ~1e-16 (used where differences of Gram entries decide a ranking).
hipError_t launch_gemm64_bf16(const GemmArgs& g, hipStream_t stream);

// ---------------------------------------------------------------- elementwise.hip
// out[c][r] = in[r][c] for a rows x cols matrix of bf16 or fp32 elements.
hipError_t launch_transpose(const void* in, void* out, int rows, int cols, int dtype, hipStream_t stream);

// Token activity (paper Sec. III-A.2): s_act[b,i] = (1/K) sum_l ||hidden[b,l,i,:] - hidden[b,l-1,i,:]||_2.
hipError_t launch_activity(const void* hidden, float* s_act, int B, int N, int d, int K, int dtype, hipStream_t stream);

enum { IN_BF16 = 0, IN_F32 = 1, IN_F64 = 2 };

// out[row] = sum_c x[row,c]^2 for rows x d; out is fp32 (accumulated in fp32) or fp64.
hipError_t launch_row_norm2(const void* x, int in_type, void* out, bool out_f64, long rows, int d, hipStream_t stream);

// dst = convert(src), n elements: bf16 -> fp32 or fp32 -> fp64.
hipError_t launch_convert(const void* src, int in_type, void* dst, bool out_f64, long n, hipStream_t stream);

// v[r,c] = sum_{p < planes} src[p*plane_stride + r*d + c] (added in plane order), then split into three
// bf16 planes hi/mid/lo with hi+mid+lo == v to ~2^-25 relative.  Output row of (r, s):
// ((r / rows_per_group) * 3 + s) * rows_per_group + r % rows_per_group.
hipError_t launch_sum_split3(const float* src, int planes, long plane_stride, long rows, int d, long rows_per_group,
                             unsigned short* out, hipStream_t stream);

// Query-aware score (paper Sec. III-A.1): s_query[b,i] = max_j L[b,i,j] / max(|e(v_i)| |e(q_j)|, 1e-30) with
// L[b,i,j] = sum_{s<planes} logits[b,i,s*T+j], |e(v_i)|^2 = sum_{t<nparts} vnorm2[(b*N+i)*nparts + t],
// |e(q_j)|^2 = qnorm2[b*T+j].  The three inputs are fp32, or fp64 when f64 is set.
hipError_t launch_cosine_max(const void* logits, int planes, const void* vnorm2, int nparts, const void* qnorm2, bool f64,
                             float* s_query, int B, int N, int T, hipStream_t stream);

// Attention-softmax relevance (variant): S is [B,H,T,N] logits (unscaled; fp32, or fp64 when f64 is set).
// Pass 1 writes per (b,h,j) the row maximum and the sum of exponentials of scale*S as a double2; pass 2
// averages the probabilities over (h,j).
// softmax_base2(f64, N): fp32 logits with N % 4 == 0 take 16-byte loads and base-2 exponentials; then both calls
// must be made with base2 = true / a `part` scratch of softmax_scratch_bytes(B, N) bytes (the statistics are kept
// in base-2 units).
bool softmax_base2(bool f64, int N);
size_t softmax_scratch_bytes(int B, int N);
hipError_t launch_softmax_stats(const void* S, bool f64, void* stats, long rows, int N, double scale, bool base2, hipStream_t stream);
hipError_t launch_softmax_mean(const void* S, bool f64, const void* stats, float* s_query, int B, int HT, int N,
                               double scale, void* part, hipStream_t stream);

// Per-image min-max normalisation and fusion (paper fusion equation):
// s_fused = lambda*minmax(s_query) + (1-lambda)*minmax(s_act);  s_act == nullptr => s_fused = minmax(s_query).
hipError_t launch_fuse(const float* s_query, const float* s_act, float* s_fused, int B, int N, float lambda,
                       hipStream_t stream);

// out[b,j,:] = X[b, idx[b,j], :]  (bit copy; row_bytes multiple of 16).
hipError_t launch_gather_rows(const void* X, const int32_t* idx, void* out, int B, int N, int k, long row_bytes,
                              hipStream_t stream);

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t stream);
hipError_t launch_fill_int(int* p, int n, int value, hipStream_t stream);

// Reproducible uniform scores for the random-selection ablation: out[b, i] = top 24 bits of
// mix64(seed * 0x9E3779B97F4A7C15 + (b << 32 | i) + 0x632BE59BD9B4E019) times 2^-24 (mix64 = SplitMix64 output function).
hipError_t launch_random_scores(float* out, int B, int N, uint32_t seed, int image0, hipStream_t stream);

// ---------------------------------------------------------------- select.hip
// Per image: positions of the m largest of scores[b, 0..n) (ties -> lower position), ascending.
// out[b,j] = map ? map[b*n + pos] : pos.   n <= 16384.
hipError_t launch_select_top(const float* scores, int B, int n, int m, const int32_t* map, int32_t* out,
                             hipStream_t stream);

// Bound of every wait of one workgroup for the others of its image (eigen-solve, greedy picks), in ticks of the
// 100 MHz wall clock; process-wide, read at launch.  ticks <= 0 restores the default of 2 s.
void set_barrier_limit_ticks(long long ticks);
long long barrier_limit_ticks();

// ---------------------------------------------------------------- eigen.hip
// One-sided block Jacobi on the rows of the symmetric PSD matrices A[b] (fp64, pitch nP = jacobi_pitch(n),
// rows/cols >= n zero).  On return the r longest rows k of A[b] are lambda_k v_k^T (shorter rows only span the rest).  `ctl` is scratch of jacobi_ctl_bytes(B), `len2` scratch of B*nP doubles.
size_t jacobi_ctl_bytes(int B);
int jacobi_pitch(int n);      // row pitch (and padded order) the solver needs: n rounded up to 64
// preset_done (optional, [B]): images whose entry is non-zero are left untouched.
// img_status (optional, [B]): set to 1 for an image whose workgroups gave up waiting for one another (its rows
// are then NaN); never cleared here.
// band (optional, [B]): largest super-block distance (32 rows each) whose pairs are visited, for matrices whose rows
// only couple to near neighbours (see launch_band_limit); nullptr or an entry that saves no rounds: every pair.
hipError_t launch_jacobi_eigen(double* A, int B, int n, int nP, int r, void* ctl, double* len2, const int* preset_done,
                               const int* band, int* img_status, hipStream_t stream);
// dmax[b] = largest distance between 32-row super-blocks at which rows of the symmetric n x n matrix H[b] couple with a
// weight of at least tol, given S[b] = H[b]^2 (pitch n, lower triangle read); n % 32 == 0.
// skip (optional, [B]): images with a non-zero entry are left out.
hipError_t launch_band_limit(const double* S, int B, int n, double tol, int* dmax, const int* skip, hipStream_t stream);
hipError_t launch_row_lengths(const double* A, int B, int rows, int pitch, long img_stride, double* lam, hipStream_t stream);
// Subspace energy (paper energy equation) from rows of the form lambda_k v_k^T: c[b,i] = sum over the r
// longest of the `rows` rows of A[b] of A[k][i]^2 / |row k|, i < n.  A[b] starts at b*img_stride, rows have
// `pitch` doubles.  `lam` is scratch of B*rows doubles.  Images with flag[b] != run_if are skipped
// (flag == nullptr: none).
hipError_t launch_subspace_energy(const double* A, int B, int rows, int n, int pitch, long img_stride, int r, double* lam,
                                  float* c, const int* flag, int run_if, hipStream_t stream);

// ---------------------------------------------------------------- subspace.hip
// Block subspace iteration for the r dominant eigenpairs of G[b] (fp64, n x n, pitch nP, left untouched).
// subspace_block: block size P for (n, r), 0 when the full solve is the better choice.
// On return ok[b] = 1 where the residual check passed; then the P rows of (*ut)[b] (pitch nP) are
// theta_k u_k^T with the r longest converged.  jacobi_ctl / jacobi_len2 as for launch_jacobi_eigen.
int subspace_block(int n, int r);
size_t subspace_workspace_bytes(int B, int n, int nP, int P);
// probe_begin / probe_end (optional): recorded around the first of the subspace_product_launches(iters)
// equal launches of the product Yt G (P x nP x nP per image).
int subspace_product_launches(int iters);
hipError_t launch_subspace_eigen(const double* G, int B, int n, int nP, int r, int P, int iters, int more_iters, void* ws, void* jacobi_ctl,
                                 double* jacobi_len2, int* ok, const double** ut, int* img_status, hipEvent_t probe_begin,
                                 hipEvent_t probe_end, hipStream_t stream);

// ---------------------------------------------------------------- greedy.hip
// Greedy residual picks (variant): pivoted Cholesky of G[b] (fp64, pitch nP; G may be overwritten with the residual
// matrix).  Lt is scratch [B][k][nP] fp64.
// order[b,t] = local position picked at step t, resid[b,t] = residual squared norm at that pick.
// nP % 64 == 0; `scratch` holds greedy_scratch_bytes(B, nP) bytes (barrier counters and per-step posts).
size_t greedy_scratch_bytes(int B, int nP);
// img_status (optional, [B]): set to 1 for an image whose workgroups gave up waiting for one another (order[b] is
// then 0..k-1 and its residuals NaN); never cleared here.
hipError_t launch_greedy(double* G, int B, int n, int nP, int k, double* Lt, int32_t* order, float* resid, void* scratch,
                         int* img_status, hipStream_t stream);
// idx_out[b,:] = sort ascending of idx_m[b, order[b,:]];  pick_out[b,t] = idx_m[b, order[b,t]] (optional).
hipError_t launch_greedy_finish(const int32_t* order, const int32_t* idx_m, int B, int M, int k, int32_t* idx_out,
                                int32_t* pick_out, hipStream_t stream);

// ---------------------------------------------------------------- stream.hip
// Streaming selection (frame by frame; not in the paper): candidates of a frame = the n_keep kept tokens, then
// the frame's m pre-selected tokens.  State pitch kcap: Z [B, kcap, row], id [B, kcap], G [B, kcap, kcap].
// idc[b, i] = id of candidate i.
hipError_t launch_stream_ids(const int32_t* id_in, const int32_t* idx_f, int32_t* idc, int B, int n_keep, int m, int kcap,
                             int id_base, hipStream_t stream);
// dst[b][i][j] = src[b][i][j], i, j < n.
hipError_t launch_copy_block(double* dst, long dpitch, long dstride, const double* src, long spitch, long sstride, int n, int B,
                             hipStream_t stream);
// G[b][j][i] = G[b][i][j] for n0 <= i < n1, j < n0.
hipError_t launch_mirror_block(double* G, long pitch, long stride, int n0, int n1, int B, hipStream_t stream);
// Next state: row j = candidate sel[b, j] (sel == nullptr: candidate j), with its id and the Gram block of the
// survivors gathered from Gc (pitch, image stride).  row_bytes % 16 == 0; in and out state must not overlap.
hipError_t launch_stream_compact(const void* Z_in, const void* X, const int32_t* idx_f, const int32_t* sel, const int32_t* idc,
                                 const double* Gc, long pitch, long stride, void* Z_out, int32_t* id_out, double* G_out, int B,
                                 int n_keep, int m, int kcap, int N, int n_out, long row_bytes, hipStream_t stream);

// ---------------------------------------------------------------- verify.hip
// Speculative verification over the vocabulary (paper Sec. II-A): zt, zd [S, L, V] target / draft logits,
// tok [S, L] drafted tokens, u_acc [S, L], u_res [S] uniforms.  n_acc[s] = accepted positions before the first
// rejection, corr[s] = correction drawn from the residual distribution there (-1 if none), alpha [S, L] optional.
size_t verify_workspace_bytes(int S, int L, int V, int dtype);
hipError_t launch_verify(const void* zt, const void* zd, const int32_t* tok, const float* u_acc, const float* u_res, int S, int L,
                         int V, int dtype, int32_t* n_acc, int32_t* corr, float* alpha, void* ws, hipStream_t stream);

// ---------------------------------------------------------------- draft.hip
// Draft-side vocabulary pass (paper Sec. III-B margin gate, Sec. III-C bonus-token candidates): zd [S, L, V] draft
// logits, tok [S, L] drafted tokens, fanout[L] (host) = F_j <= F0 <= 32.  margin, gate [S, L]; cand [S, L, F0]
// (-1 beyond F_j; may be NULL when F0 == 0).
int draft_chunks(int V);
int draft_max_vocab();
size_t draft_workspace_bytes(int S, int L, int V);
hipError_t launch_draft(const void* zd, const int32_t* tok, int S, int L, int V, int dtype, int F0, const int* fanout, float gamma,
                        float* margin, int32_t* gate, int32_t* cand, void* ws, hipStream_t stream);

}  // namespace covspec
