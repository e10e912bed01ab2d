// C ABI of the visual-token-reduction library: argument validation, workspace
// carving and the launch sequence of paper Sec. III-A (score, fuse, pre-select,
// low-rank energy, keep, gather).  No allocation, no synchronisation, no global state.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdio.h>

#include <atomic>

#include "../../include/covspec.h"
#include "kernels.h"

using namespace covspec;

namespace {

constexpr int kMaxTokens = 16384;
constexpr int kMaxPreselect = 4096;
constexpr int kMaxActLayers = 8;
constexpr int kSubspaceIters = 12;       // steps before the first residual check (the workloads pass it with a factor >= 10 to spare)
constexpr int kSubspaceMoreIters = 4;    // further steps for the images that fail it, before the full solve

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Plan {
  int B, N, d, T, H, K, dtype, rel, lr, M, r, k;
  float lambda;
  uint32_t seed;
  int image0;     // index of the first image in the caller's batch (ragged batches run as several calls)
  int esz;        // bytes per stored element
  int planes;     // bf16: 3 split planes of the folded query matrix, fp32: 1
  int nparts;     // per-token partial sums of |e(v)|^2 written by the projection GEMM
  int nP;         // Gram pitch (padded order of the eigen-solve)
  // workspace offsets (bytes)
  size_t wqT, wkT, Eq, qn2, Eq3, G3raw, G3, vn2p, logits, Ev, S, stats, smean, sq, sa, sf;
  size_t idxm, Awork, ctl, lam, c, Lt, order, resid, gscr, sub, ok, status;
  int P;          // block size of the subspace iteration (0: full Jacobi solve)
  size_t total;
};

int resolve(const covspec_params* p, int* k_, int* M_, int* r_) {
  if (!p) return COVSPEC_INVALID_ARG;
  if (p->n_tokens < 1 || p->keep_k < 0 || p->preselect_m < 0 || p->rank_r < 0) return COVSPEC_INVALID_ARG;
  const long N = p->n_tokens;
  long k = p->keep_k;
  if (k == 0) {
    if (!(p->keep_ratio > 0.f) || !(p->keep_ratio <= 1.f)) return COVSPEC_INVALID_ARG;
    k = (long)floor((double)p->keep_ratio * (double)N + 0.5);
    if (k < 1) k = 1;
    if (k > N) k = N;
  }
  long M = p->preselect_m > 0 ? p->preselect_m : (2 * k < N ? 2 * k : N);
  if (p->keep_k == 0 && k > M) k = M;
  long r = p->rank_r > 0 ? p->rank_r : (k / 2 > 1 ? k / 2 : 1);
  if (M > N || k > M || k < 1) return COVSPEC_INVALID_ARG;
  *k_ = (int)k; *M_ = (int)M; *r_ = (int)r;
  return COVSPEC_OK;
}

int make_plan(const covspec_params* p, Plan* pl) {
  if (!p) return COVSPEC_INVALID_ARG;
  if (p->batch < 1 || p->n_tokens < 1 || p->d_model < 1 || p->n_query < 1 || p->n_heads < 1) return COVSPEC_INVALID_ARG;
  if (p->d_model % p->n_heads != 0) return COVSPEC_INVALID_ARG;
  if (p->n_act_layers < 0) return COVSPEC_INVALID_ARG;
  if (p->dtype != COVSPEC_FP32 && p->dtype != COVSPEC_BF16) return COVSPEC_INVALID_ARG;
  if (p->rel_mode != COVSPEC_REL_COSINE_MAX && p->rel_mode != COVSPEC_REL_ATTN_SOFTMAX) return COVSPEC_INVALID_ARG;
  if (p->lr_mode < COVSPEC_LR_ENERGY_TOPK || p->lr_mode > COVSPEC_LR_RANDOM) return COVSPEC_INVALID_ARG;
  if (!(p->lambda >= 0.f) || !(p->lambda <= 1.f)) return COVSPEC_INVALID_ARG;
  int k, M, r;
  int st = resolve(p, &k, &M, &r);
  if (st != COVSPEC_OK) return st;
  const int mind = M < p->d_model ? M : p->d_model;
  if (p->lr_mode == COVSPEC_LR_ENERGY_TOPK && (r < 1 || r >= mind)) return COVSPEC_INVALID_ARG;
  // limits of the kernels
  const bool lowrank = p->lr_mode == COVSPEC_LR_ENERGY_TOPK || p->lr_mode == COVSPEC_LR_GREEDY_RESIDUAL;
  if (p->n_tokens > kMaxTokens || (lowrank && M > kMaxPreselect) || p->n_act_layers > kMaxActLayers) return COVSPEC_UNSUPPORTED;
  if (p->d_model % (p->dtype == COVSPEC_BF16 ? 8 : 4) != 0) return COVSPEC_UNSUPPORTED;
  if (p->rel_mode == COVSPEC_REL_ATTN_SOFTMAX && (p->d_model / p->n_heads) % 4 != 0) return COVSPEC_UNSUPPORTED;
  if ((long)p->batch * p->n_tokens > 0x3fffffffL || (long)p->batch * p->n_query > 0x3fffffffL) return COVSPEC_UNSUPPORTED;

  Plan& q = *pl;
  q.B = p->batch; q.N = p->n_tokens; q.d = p->d_model; q.T = p->n_query; q.H = p->n_heads; q.K = p->n_act_layers;
  q.dtype = p->dtype; q.rel = p->rel_mode; q.lr = p->lr_mode; q.M = M; q.r = r; q.k = k; q.lambda = p->lambda; q.seed = p->seed; q.image0 = 0;
  q.esz = p->dtype == COVSPEC_BF16 ? 2 : 4;
  q.planes = p->dtype == COVSPEC_BF16 ? 3 : 1;
  q.nparts = p->dtype == COVSPEC_BF16 ? gemm_tiles_n(q.d) : gemm64_tiles_n(q.d);
  const size_t fsz = p->dtype == COVSPEC_BF16 ? 4 : 8;  // bytes per intermediate value
  q.nP = jacobi_pitch(M);

  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  const size_t B = q.B, N = q.N, d = q.d, T = q.T, BT = B * T, BN = B * N;
  q.wqT = q.wkT = q.Eq = q.qn2 = 0;
  q.Eq3 = q.G3raw = q.G3 = q.vn2p = q.logits = q.Ev = q.S = q.stats = q.smean = 0;
  // the random-selection ablation uses no scores; covspec_score with that mode still works on its own
  // workspace request, so the score buffers are always part of the plan
  q.wqT = take(d * d * q.esz);
  q.wkT = take(d * d * q.esz);
  q.Eq = take(BT * d * fsz);
  q.qn2 = take(BT * fsz);
  if (q.rel == COVSPEC_REL_COSINE_MAX) {
    if (q.dtype == COVSPEC_BF16) q.Eq3 = take(3 * BT * d * 2);
    q.G3raw = take((size_t)q.planes * BT * d * fsz);
    if (q.dtype == COVSPEC_BF16) q.G3 = take(3 * BT * d * 2);
    q.vn2p = take(BN * q.nparts * fsz);
    q.logits = take(BN * q.planes * T * fsz);
  } else {
    q.Ev = take(BN * d * fsz);
    q.S = take(B * q.H * T * N * fsz);
    q.stats = take(B * q.H * T * 16);
    if (softmax_base2(q.dtype == COVSPEC_FP32, q.N)) q.smean = take(softmax_scratch_bytes(q.B, q.N));
  }
  q.sq = take(BN * 4);
  q.sa = take(BN * 4);
  q.sf = take(BN * 4);
  q.idxm = take(B * M * 4);
  q.status = take(B * 4);       // per image: 1 when the bounded wait of a multi-workgroup kernel gave up
  q.Awork = q.ctl = q.lam = q.c = q.sub = q.ok = 0;
  q.P = 0;
  if (lowrank) {
    q.Awork = take(B * (size_t)q.nP * q.nP * 8);
    q.ctl = take(jacobi_ctl_bytes(q.B));
    q.lam = take(B * q.nP * 8);
    q.c = take(B * M * 4);
    q.P = (q.lr == COVSPEC_LR_ENERGY_TOPK) ? subspace_block(M, r) : 0;
    q.sub = take(subspace_workspace_bytes(q.B, M, q.nP, q.P));
    q.ok = take(B * 4);
  }
  q.Lt = q.order = q.resid = q.gscr = 0;
  if (q.lr == COVSPEC_LR_GREEDY_RESIDUAL) {
    q.Lt = take(B * (size_t)k * q.nP * 8);
    q.order = take(B * k * 4);
    q.resid = take(B * k * 4);
    q.gscr = take(greedy_scratch_bytes(q.B, q.nP));
  }
  q.total = off;
  return COVSPEC_OK;
}

// What failed last on this host thread, for covspec_last_error().
thread_local char g_last_error[256] = "";

inline void note_error(const char* what, hipError_t e) {
  snprintf(g_last_error, sizeof(g_last_error), "%s: %s", hipGetErrorName(e), what);
}

// The launchers report through hipGetLastError(), which also returns an error that some EARLIER runtime call
// of this thread left behind (another library's, a query that answered "not ready").  Every entry point that
// launches therefore discards what is pending before its first launch.
inline void discard_pending_error() { (void)hipGetLastError(); }

#define HIPCHK(expr)                                \
  do {                                              \
    hipError_t e__ = (expr);                        \
    if (e__ != hipSuccess) {                        \
      note_error(#expr, e__);                       \
      return COVSPEC_HIP_ERROR;                     \
    }                                               \
  } while (0)

template <typename T>
inline T* at(void* ws, size_t off) { return (T*)((char*)ws + off); }

// Optional per-stage timing: records the caller's events on the work stream at stage boundaries.
struct StageMarks {
  hipEvent_t* ev = nullptr;
  hipStream_t st = nullptr;
  bool ok = true;
  void mark(int stage) {
    if (!ev) return;
    const hipError_t e = hipEventRecord(ev[stage], st);
    if (e != hipSuccess) { ok = false; note_error("hipEventRecord of a stage event", e); }
  }
};

int check_ws(const Plan& pl, void* ws, size_t bytes) {
  if (!ws || ((uintptr_t)ws & 255u)) return COVSPEC_INVALID_ARG;
  if (bytes < pl.total) return COVSPEC_WORKSPACE_TOO_SMALL;
  return COVSPEC_OK;
}

// ---- scores: paper Sec. III-A.1 (query-aware), III-A.2 (activity), fusion equation
//
// bf16 storage: contractions on the bf16 MFMA with fp32 accumulation, fp32 intermediates.
// fp32 storage: every contraction and intermediate in fp64 (see gemm64.hip).
int run_score(const Plan& q, const void* X, const void* hidden, const void* Q, const void* Wq, const void* Wk,
              float* s_query, float* s_act, float* s_fused, void* ws, hipStream_t st, StageMarks& marks) {
  const long B = q.B, N = q.N, d = q.d, T = q.T, BT = B * T, BN = B * N;
  const bool f64 = q.dtype == COVSPEC_FP32;
  const int in_x = f64 ? IN_F32 : IN_BF16;      // storage type of X, Q, W
  const int in_mid = f64 ? IN_F64 : IN_F32;     // type of the intermediates
  void* Eq = at<void>(ws, q.Eq);
  void* qn2 = at<void>(ws, q.qn2);
  float* sq = s_query ? s_query : at<float>(ws, q.sq);
  float* sf = s_fused ? s_fused : at<float>(ws, q.sf);
  const bool has_act = hidden != nullptr && q.K > 0;
  float* sa = has_act ? (s_act ? s_act : at<float>(ws, q.sa)) : nullptr;
  auto gemm = [&](const GemmArgs& g, bool a_mid, bool b_mid) -> hipError_t {
    // a_mid / b_mid: operand is an intermediate (fp64 on the fp64 path) rather than a stored input
    return f64 ? launch_gemm64_nt(g, a_mid, b_mid, st) : launch_gemm_nt(g, DT_BF16, st);
  };

  // A score whose weight in the fusion is zero is computed only if the caller asked for it (selector ablations,
  // Table II: query-only is lambda = 1, activity-only lambda = 0); 0 * score adds an exact zero for finite scores.
  const bool need_q = s_query != nullptr || q.lambda > 0.f || !has_act;
  const bool need_a = has_act && (s_act != nullptr || q.lambda < 1.f);

  marks.mark(COVSPEC_STAGE_QUERY_SIDE);
  auto query_scores = [&]() -> int {
  // e(q) = q Wq
  if (Wq) {
    HIPCHK(launch_transpose(Wq, at<void>(ws, q.wqT), q.d, q.d, q.dtype, st));
    GemmArgs g;
    g.A = Q; g.B = at<void>(ws, q.wqT); g.C = Eq; g.M = (int)BT; g.N = q.d; g.K = q.d; g.lda = d; g.ldb = d; g.ldc = d;
    g.epilogue = f64 ? EPI_STORE_F64 : EPI_STORE_F32;
    HIPCHK(gemm(g, false, false));
  } else {
    HIPCHK(launch_convert(Q, in_x, Eq, f64, BT * d, st));
  }
  if (Wk) HIPCHK(launch_transpose(Wk, at<void>(ws, q.wkT), q.d, q.d, q.dtype, st));

  if (q.rel == COVSPEC_REL_COSINE_MAX) {
    HIPCHK(launch_row_norm2(Eq, in_mid, qn2, f64, BT, q.d, st));
    // fold Wk into the query side: <x Wk, e(q)> = <x, Wk e(q)^T>; the token side then only needs |x Wk|^2
    const void* Gq;  // per image [planes*T, d]
    void* vn2 = at<void>(ws, q.vn2p);
    int nparts;
    if (Wk) {
      void* Graw = at<void>(ws, q.G3raw);
      GemmArgs g;
      g.B = Wk; g.C = Graw; g.N = q.d; g.K = q.d; g.lda = d; g.ldb = d; g.ldc = d;
      if (!f64) {
        HIPCHK(launch_sum_split3((const float*)Eq, 1, 0, BT, q.d, BT, at<unsigned short>(ws, q.Eq3), st));
        g.A = at<void>(ws, q.Eq3); g.M = (int)(3 * BT);
        HIPCHK(launch_gemm_nt(g, DT_BF16, st));
        HIPCHK(launch_sum_split3((const float*)Graw, 3, BT * d, BT, q.d, T, at<unsigned short>(ws, q.G3), st));
        Gq = at<void>(ws, q.G3);
      } else {
        g.A = Eq; g.M = (int)BT; g.epilogue = EPI_STORE_F64;
        HIPCHK(launch_gemm64_nt(g, true, false, st));
        Gq = Graw;
      }
      marks.mark(COVSPEC_STAGE_TOKEN_PROJECTION);
      GemmArgs n;
      n.A = X; n.B = at<void>(ws, q.wkT); n.C = vn2; n.M = (int)BN; n.N = q.d; n.K = q.d; n.lda = d; n.ldb = d;
      n.ldc = q.nparts; n.epilogue = EPI_ROWNORM2;
      HIPCHK(gemm(n, false, false));
      nparts = q.nparts;
    } else {
      if (!f64) {
        HIPCHK(launch_sum_split3((const float*)Eq, 1, 0, BT, q.d, T, at<unsigned short>(ws, q.G3), st));
        Gq = at<void>(ws, q.G3);
      } else {
        Gq = Eq;
      }
      marks.mark(COVSPEC_STAGE_TOKEN_PROJECTION);
      HIPCHK(launch_row_norm2(X, in_x, vn2, f64, BN, q.d, st));
      nparts = 1;
    }
    marks.mark(COVSPEC_STAGE_RELEVANCE);
    void* logits = at<void>(ws, q.logits);
    GemmArgs l;
    l.A = X; l.B = Gq; l.C = logits; l.M = q.N; l.N = q.planes * q.T; l.K = q.d; l.lda = d; l.ldb = d; l.ldc = q.planes * T;
    l.batch = q.B; l.strideA = N * d; l.strideB = (long)q.planes * T * d; l.strideC = N * q.planes * T;
    l.epilogue = f64 ? EPI_STORE_F64 : EPI_STORE_F32;
    HIPCHK(gemm(l, false, true));
    HIPCHK(launch_cosine_max(logits, q.planes, vn2, nparts, qn2, f64, sq, q.B, q.N, q.T, st));
  } else {
    // variant: e(v) materialised, per-head logits, softmax over the visual tokens
    marks.mark(COVSPEC_STAGE_TOKEN_PROJECTION);
    void* Ev = at<void>(ws, q.Ev);
    if (Wk) {
      GemmArgs g;
      g.A = X; g.B = at<void>(ws, q.wkT); g.C = Ev; g.M = (int)BN; g.N = q.d; g.K = q.d; g.lda = d; g.ldb = d; g.ldc = d;
      g.epilogue = f64 ? EPI_STORE_F64 : EPI_STORE_F32;
      HIPCHK(gemm(g, false, false));
    } else {
      HIPCHK(launch_convert(X, in_x, Ev, f64, BN * d, st));
    }
    marks.mark(COVSPEC_STAGE_RELEVANCE);
    const int dh = q.d / q.H;
    void* S = at<void>(ws, q.S);
    GemmArgs g;
    g.A = Eq; g.B = Ev; g.C = S; g.M = q.T; g.N = q.N; g.K = dh; g.lda = d; g.ldb = d; g.ldc = N;
    g.batch = q.B * q.H; g.batch_inner = q.H;
    g.strideA = T * d; g.strideA2 = dh; g.strideB = N * d; g.strideB2 = dh; g.strideC = (long)q.H * T * N; g.strideC2 = T * N;
    g.epilogue = f64 ? EPI_STORE_F64 : EPI_STORE_F32;
    HIPCHK(f64 ? launch_gemm64_nt(g, true, true, st) : launch_gemm_nt(g, DT_F32, st));
    const double scale = 1.0 / sqrt((double)dh);
    void* stats = at<void>(ws, q.stats);
    const bool base2 = softmax_base2(f64, q.N);
    HIPCHK(launch_softmax_stats(S, f64, stats, B * q.H * T, q.N, scale, base2, st));
    HIPCHK(launch_softmax_mean(S, f64, stats, sq, q.B, q.H * q.T, q.N, scale, base2 ? at<void>(ws, q.smean) : nullptr, st));
  }
  return COVSPEC_OK;
  };
  if (need_q) {
    const int rc = query_scores();
    if (rc != COVSPEC_OK) return rc;
  } else {
    marks.mark(COVSPEC_STAGE_TOKEN_PROJECTION);
    marks.mark(COVSPEC_STAGE_RELEVANCE);
  }

  marks.mark(COVSPEC_STAGE_ACTIVITY);
  if (need_a) HIPCHK(launch_activity(hidden, sa, q.B, q.N, q.d, q.K, q.dtype, st));
  marks.mark(COVSPEC_STAGE_FUSE);
  // with one score left the fused score is that score, min-max normalised
  if (need_q) HIPCHK(launch_fuse(sq, need_a ? sa : nullptr, sf, q.B, q.N, q.lambda, st));
  else HIPCHK(launch_fuse(sa, nullptr, sf, q.B, q.N, q.lambda, st));
  return COVSPEC_OK;
}

// ---- selection: paper Sec. III-A.3
int run_select(const Plan& q, const void* X, const float* s_fused, int32_t* idx_out, float* c_out, int32_t* idx_m_out,
               int32_t* pick_order_out, float* resid_out, void* ws, hipStream_t st, StageMarks& marks) {
  const long N = q.N, d = q.d;
  marks.mark(COVSPEC_STAGE_PRESELECT);
  int* img_status = at<int>(ws, q.status);
  HIPCHK(launch_fill_int(img_status, q.B, 0, st));
  if (q.lr == COVSPEC_LR_SCORE_TOPK || q.lr == COVSPEC_LR_RANDOM) {
    // selector ablations (Table II; Sec. III-A.3, first sentence): one ranking, no low-rank stage
    const float* rank_by = s_fused;
    if (q.lr == COVSPEC_LR_RANDOM) {
      float* u = at<float>(ws, q.sf);   // the fused-score buffer is free: this mode uses no scores
      HIPCHK(launch_random_scores(u, q.B, q.N, q.seed, q.image0, st));
      rank_by = u;
    } else if (idx_m_out) {
      HIPCHK(launch_select_top(s_fused, q.B, q.N, q.M, nullptr, idx_m_out, st));
    }
    marks.mark(COVSPEC_STAGE_GRAM);
    marks.mark(COVSPEC_STAGE_LOWRANK);
    marks.mark(COVSPEC_STAGE_KEEP);
    HIPCHK(launch_select_top(rank_by, q.B, q.N, q.k, nullptr, idx_out, st));
    marks.mark(COVSPEC_PROBE_BEGIN);
    marks.mark(COVSPEC_PROBE_END);
    return COVSPEC_OK;
  }
  int32_t* idxm = idx_m_out ? idx_m_out : at<int32_t>(ws, q.idxm);
  HIPCHK(launch_select_top(s_fused, q.B, q.N, q.M, nullptr, idxm, st));

  // token Gram matrix of the pre-selected rows, fp64, zero-padded to the pitch
  marks.mark(COVSPEC_STAGE_GRAM);
  double* A = at<double>(ws, q.Awork);
  HIPCHK(launch_fill_zero(A, (size_t)q.B * q.nP * q.nP * 8, st));
  GemmArgs g;
  g.A = X; g.B = X; g.C = A; g.M = q.M; g.N = q.M; g.K = q.d; g.lda = d; g.ldb = d; g.ldc = q.nP;
  g.batch = q.B; g.strideA = N * d; g.strideB = N * d; g.strideC = (long)q.nP * q.nP;
  g.gatherA = idxm; g.gatherB = idxm; g.gstrideA = q.M; g.gstrideB = q.M;
  g.epilogue = EPI_STORE_F64;
  // The greedy variant ranks residuals, i.e. differences of Gram entries that shrink far below the
  // entries themselves, so its Gram matrix is accumulated in fp64; the energy ranking is not a
  // cancellation and takes the bf16 MFMA with fp32 partial sums flushed into fp64.
  if (q.dtype == COVSPEC_FP32) HIPCHK(launch_gemm64_nt(g, false, false, st));
  else if (q.lr == COVSPEC_LR_GREEDY_RESIDUAL) {
    g.lower_only = true;      // Z Z^T is symmetric: the tiles above the diagonal are the transposes of those below
    g.mirror = true;
    HIPCHK(launch_gemm64_bf16(g, st));
  }
  else {
    g.lower_only = true;
    g.mirror = true;
    HIPCHK(launch_gemm_nt(g, DT_BF16, st));
  }

  bool probed = false;
  if (q.lr == COVSPEC_LR_ENERGY_TOPK) {
    float* c = c_out ? c_out : at<float>(ws, q.c);
    marks.mark(COVSPEC_STAGE_LOWRANK);
    if (q.P > 0) {
      // r dominant eigenpairs by block subspace iteration; images whose residual check fails fall back to
      // the full Jacobi solve (which leaves the others untouched)
      int* ok = at<int>(ws, q.ok);
      const double* Ut = nullptr;
      HIPCHK(launch_subspace_eigen(A, q.B, q.M, q.nP, q.r, q.P, kSubspaceIters, kSubspaceMoreIters, at<void>(ws, q.sub), at<void>(ws, q.ctl),
                                   at<double>(ws, q.lam), ok, &Ut, img_status, marks.ev ? marks.ev[COVSPEC_PROBE_BEGIN] : nullptr,
                                   marks.ev ? marks.ev[COVSPEC_PROBE_END] : nullptr, st));
      probed = true;
      HIPCHK(launch_jacobi_eigen(A, q.B, q.M, q.nP, q.r, at<void>(ws, q.ctl), at<double>(ws, q.lam), ok, nullptr, img_status, st));
      marks.mark(COVSPEC_STAGE_KEEP);
      HIPCHK(launch_subspace_energy(Ut, q.B, q.P, q.M, q.nP, (long)q.P * q.nP, q.r, at<double>(ws, q.lam), c, ok, 1, st));
      HIPCHK(launch_subspace_energy(A, q.B, q.M, q.M, q.nP, (long)q.nP * q.nP, q.r, at<double>(ws, q.lam), c, ok, 0, st));
    } else {
      HIPCHK(launch_jacobi_eigen(A, q.B, q.M, q.nP, q.r, at<void>(ws, q.ctl), at<double>(ws, q.lam), nullptr, nullptr, img_status, st));
      marks.mark(COVSPEC_STAGE_KEEP);
      HIPCHK(launch_subspace_energy(A, q.B, q.M, q.M, q.nP, (long)q.nP * q.nP, q.r, at<double>(ws, q.lam), c, nullptr, 0, st));
    }
    HIPCHK(launch_select_top(c, q.B, q.M, q.k, idxm, idx_out, st));
  } else {
    int32_t* order = at<int32_t>(ws, q.order);
    float* resid = resid_out ? resid_out : at<float>(ws, q.resid);
    marks.mark(COVSPEC_STAGE_LOWRANK);
    HIPCHK(launch_greedy(A, q.B, q.M, q.nP, q.k, at<double>(ws, q.Lt), order, resid, at<void>(ws, q.gscr), img_status, st));
    marks.mark(COVSPEC_STAGE_KEEP);
    HIPCHK(launch_greedy_finish(order, idxm, q.B, q.M, q.k, idx_out, pick_order_out, st));
  }
  if (!probed) {
    marks.mark(COVSPEC_PROBE_BEGIN);
    marks.mark(COVSPEC_PROBE_END);
  }
  return COVSPEC_OK;
}

// ---- streaming selection (frame by frame; each frame is one low-rank step of Sec. III-A.3 on the candidates)
struct StreamPlan {
  int B, N, d, dtype, M, k, r, cap, nP, esz, P;
  size_t idxf, idc, sel, Gc, A, ctl, lam, c, sub, ok, total;
};

int make_stream_plan(const covspec_stream_params* p, StreamPlan* pl) {
  if (!p) return COVSPEC_INVALID_ARG;
  if (p->batch < 1 || p->n_frame < 1 || p->d_model < 1 || p->keep_k < 1) return COVSPEC_INVALID_ARG;
  if (p->dtype != COVSPEC_FP32 && p->dtype != COVSPEC_BF16) return COVSPEC_INVALID_ARG;
  if (p->frame_m < 1 || p->frame_m > p->n_frame) return COVSPEC_INVALID_ARG;
  const int mind = p->keep_k < p->d_model ? p->keep_k : p->d_model;
  if (p->rank_r < 1 || p->rank_r >= mind) return COVSPEC_INVALID_ARG;
  if ((long)p->keep_k + p->frame_m > kMaxPreselect || p->n_frame > kMaxTokens) return COVSPEC_UNSUPPORTED;
  if (p->d_model % (p->dtype == COVSPEC_BF16 ? 8 : 4) != 0) return COVSPEC_UNSUPPORTED;
  if ((long)p->batch * p->n_frame > 0x3fffffffL) return COVSPEC_UNSUPPORTED;
  StreamPlan& q = *pl;
  q.B = p->batch; q.N = p->n_frame; q.d = p->d_model; q.dtype = p->dtype; q.M = p->frame_m; q.k = p->keep_k; q.r = p->rank_r;
  q.cap = q.k + q.M;
  q.nP = jacobi_pitch(q.cap);
  q.esz = q.dtype == COVSPEC_BF16 ? 2 : 4;
  q.P = subspace_block(q.cap, q.r);      // the largest candidate count decides: a smaller one never needs more
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  const size_t B = q.B;
  q.idxf = take(B * q.M * 4);
  q.idc = take(B * q.cap * 4);
  q.sel = take(B * q.k * 4);
  q.Gc = take(B * (size_t)q.nP * q.nP * 8);
  q.A = take(B * (size_t)q.nP * q.nP * 8);
  q.ctl = take(jacobi_ctl_bytes(q.B));
  q.lam = take(B * q.nP * 8);
  q.c = take(B * q.cap * 4);
  q.sub = take(subspace_workspace_bytes(q.B, q.cap, q.nP, q.P));
  q.ok = take(B * 4);
  q.total = off;
  return COVSPEC_OK;
}

}  // namespace

// A ragged batch is worked off as runs of consecutive images of equal shape, each run one dense call.
struct RaggedRun { int first, count, N, T; long tok0, qry0, kept0; int k; };

// Walks the runs; fn(run, params of the run) returns a status.  keep_k_out (optional) receives k per image.
template <typename F>
static int ragged_walk(const covspec_params* p, const covspec_ragged* r, int32_t* keep_k_out, F fn) {
  if (!p || !r || r->n_images < 1 || !r->n_tokens || !r->n_query) return COVSPEC_INVALID_ARG;
  long tok0 = 0, qry0 = 0, kept0 = 0;
  int b = 0;
  while (b < r->n_images) {
    int e = b + 1;
    while (e < r->n_images && r->n_tokens[e] == r->n_tokens[b] && r->n_query[e] == r->n_query[b]) ++e;
    covspec_params q = *p;
    q.batch = e - b;
    q.n_tokens = r->n_tokens[b];
    q.n_query = r->n_query[b];
    Plan pl;
    int st = make_plan(&q, &pl);
    if (st != COVSPEC_OK) return st;
    RaggedRun run = {b, e - b, pl.N, pl.T, tok0, qry0, kept0, pl.k};
    if (keep_k_out)
      for (int i = b; i < e; ++i) keep_k_out[i] = pl.k;
    if ((st = fn(run, q, pl)) != COVSPEC_OK) return st;
    tok0 += (long)run.count * pl.N;
    qry0 += (long)run.count * pl.T;
    kept0 += (long)run.count * pl.k;
    b = e;
  }
  return COVSPEC_OK;
}

extern "C" {

size_t covspec_workspace_size(const covspec_params* p) {
  Plan pl;
  if (make_plan(p, &pl) != COVSPEC_OK) return 0;
  return pl.total;
}

int covspec_resolve(const covspec_params* p, int32_t* keep_k, int32_t* preselect_m, int32_t* rank_r) {
  Plan pl;
  int st = make_plan(p, &pl);
  if (st != COVSPEC_OK) return st;
  if (keep_k) *keep_k = pl.k;
  if (preselect_m) *preselect_m = pl.M;
  if (rank_r) *rank_r = pl.r;
  return COVSPEC_OK;
}

int covspec_score(const covspec_params* p, const void* X, const void* hidden, const void* Q, const void* Wq,
                  const void* Wk, float* s_query, float* s_act, float* s_fused, void* workspace, size_t workspace_bytes,
                  covspec_stream_t stream) {
  Plan pl;
  int st = make_plan(p, &pl);
  if (st != COVSPEC_OK) return st;
  if (!X || !Q) return COVSPEC_INVALID_ARG;
  if ((st = check_ws(pl, workspace, workspace_bytes)) != COVSPEC_OK) return st;
  discard_pending_error();
  StageMarks none;
  return run_score(pl, X, hidden, Q, Wq, Wk, s_query, s_act, s_fused, workspace, (hipStream_t)stream, none);
}

int covspec_select(const covspec_params* p, const void* X, const float* s_fused, int32_t* idx_out, float* c_out,
                   int32_t* idx_m_out, int32_t* pick_order_out, float* resid_out, void* workspace,
                   size_t workspace_bytes, covspec_stream_t stream) {
  Plan pl;
  int st = make_plan(p, &pl);
  if (st != COVSPEC_OK) return st;
  if (!X || !idx_out || (!s_fused && pl.lr != COVSPEC_LR_RANDOM)) return COVSPEC_INVALID_ARG;
  if ((st = check_ws(pl, workspace, workspace_bytes)) != COVSPEC_OK) return st;
  discard_pending_error();
  StageMarks none;
  return run_select(pl, X, s_fused, idx_out, c_out, idx_m_out, pick_order_out, resid_out, workspace, (hipStream_t)stream, none);
}

static int reduce_impl(const covspec_params* p, const void* X, const void* hidden, const void* Q, const void* Wq,
                       const void* Wk, int32_t* idx_out, void* tokens_out, void* workspace, size_t workspace_bytes,
                       hipStream_t s, StageMarks& marks, int image0 = 0) {
  Plan pl;
  int st = make_plan(p, &pl);
  if (st != COVSPEC_OK) return st;
  pl.image0 = image0;
  if (!X || !Q || !idx_out || !tokens_out) return COVSPEC_INVALID_ARG;
  if ((st = check_ws(pl, workspace, workspace_bytes)) != COVSPEC_OK) return st;
  discard_pending_error();
  float* sf = at<float>(workspace, pl.sf);
  if (pl.lr == COVSPEC_LR_RANDOM) {
    for (int e = COVSPEC_STAGE_QUERY_SIDE; e <= COVSPEC_STAGE_FUSE; ++e) marks.mark(e);   // no scores in this mode
  } else {
    st = run_score(pl, X, hidden, Q, Wq, Wk, nullptr, nullptr, sf, workspace, s, marks);
    if (st != COVSPEC_OK) return st;
  }
  st = run_select(pl, X, sf, idx_out, nullptr, nullptr, nullptr, nullptr, workspace, s, marks);
  if (st != COVSPEC_OK) return st;
  marks.mark(COVSPEC_STAGE_GATHER);
  HIPCHK(launch_gather_rows(X, idx_out, tokens_out, pl.B, pl.N, pl.k, (long)pl.d * pl.esz, s));
  marks.mark(COVSPEC_STAGE_END);
  return marks.ok ? COVSPEC_OK : COVSPEC_HIP_ERROR;
}

int covspec_reduce(const covspec_params* p, const void* X, const void* hidden, const void* Q, const void* Wq,
                   const void* Wk, int32_t* idx_out, void* tokens_out, void* workspace, size_t workspace_bytes,
                   covspec_stream_t stream) {
  StageMarks none;
  return reduce_impl(p, X, hidden, Q, Wq, Wk, idx_out, tokens_out, workspace, workspace_bytes, (hipStream_t)stream, none);
}

int covspec_reduce_staged(const covspec_params* p, const void* X, const void* hidden, const void* Q, const void* Wq,
                          const void* Wk, int32_t* idx_out, void* tokens_out, void* workspace, size_t workspace_bytes,
                          covspec_stream_t stream, void* const* stage_events) {
  if (!stage_events) return COVSPEC_INVALID_ARG;
  for (int i = 0; i < COVSPEC_NUM_STAGE_EVENTS; ++i)
    if (!stage_events[i]) return COVSPEC_INVALID_ARG;
  StageMarks marks;
  marks.ev = (hipEvent_t*)stage_events;
  marks.st = (hipStream_t)stream;
  return reduce_impl(p, X, hidden, Q, Wq, Wk, idx_out, tokens_out, workspace, workspace_bytes, (hipStream_t)stream, marks);
}

int covspec_ragged_resolve(const covspec_params* p, const covspec_ragged* r, int32_t* keep_k_out, int32_t* n_runs_out) {
  int runs = 0;
  const int st = ragged_walk(p, r, keep_k_out, [&](const RaggedRun&, const covspec_params&, const Plan&) { ++runs; return (int)COVSPEC_OK; });
  if (st == COVSPEC_OK && n_runs_out) *n_runs_out = runs;
  return st;
}

size_t covspec_ragged_workspace_size(const covspec_params* p, const covspec_ragged* r, int32_t n_streams) {
  if (n_streams < 1 || n_streams > COVSPEC_MAX_CONCURRENT_CALLS) return 0;
  size_t most = 0;
  const int st = ragged_walk(p, r, nullptr, [&](const RaggedRun&, const covspec_params&, const Plan& pl) {
    if (pl.total > most) most = pl.total;
    return (int)COVSPEC_OK;
  });
  return st == COVSPEC_OK ? align_up(most, 256) * (size_t)n_streams : 0;
}

int covspec_reduce_ragged(const covspec_params* p, const covspec_ragged* r, const void* X, const void* hidden, const void* Q,
                          const void* Wq, const void* Wk, int32_t* idx_out, void* tokens_out, void* workspace,
                          size_t workspace_bytes, const covspec_stream_t* streams, int32_t n_streams) {
  if (n_streams < 1 || n_streams > COVSPEC_MAX_CONCURRENT_CALLS || !streams) return COVSPEC_INVALID_ARG;
  if (!X || !Q || !idx_out || !tokens_out || !workspace || ((uintptr_t)workspace & 255u)) return COVSPEC_INVALID_ARG;
  const size_t need = covspec_ragged_workspace_size(p, r, n_streams);
  if (need == 0) {   // report why
    const int st = ragged_walk(p, r, nullptr, [](const RaggedRun&, const covspec_params&, const Plan&) { return (int)COVSPEC_OK; });
    return st != COVSPEC_OK ? st : COVSPEC_INVALID_ARG;
  }
  if (workspace_bytes < need) return COVSPEC_WORKSPACE_TOO_SMALL;
  const size_t slice = need / (size_t)n_streams;
  const size_t esz = p->dtype == COVSPEC_BF16 ? 2 : 4;
  const size_t d = (size_t)p->d_model, K1 = (size_t)p->n_act_layers + 1;
  int run_no = 0;
  return ragged_walk(p, r, nullptr, [&](const RaggedRun& run, const covspec_params& q, const Plan&) {
    const int slot = run_no++ % n_streams;
    StageMarks none;
    const char* Xr = (const char*)X + (size_t)run.tok0 * d * esz;
    const char* Hr = hidden ? (const char*)hidden + (size_t)run.tok0 * K1 * d * esz : nullptr;
    const char* Qr = (const char*)Q + (size_t)run.qry0 * d * esz;
    return reduce_impl(&q, Xr, Hr, Qr, Wq, Wk, idx_out + run.kept0, (char*)tokens_out + (size_t)run.kept0 * d * esz,
                       (char*)workspace + (size_t)slot * slice, slice, (hipStream_t)streams[slot], none, run.first);
  });
}

int covspec_lowrank_path(const covspec_params* p, const void* workspace, int32_t* path_out, covspec_stream_t stream) {
  Plan pl;
  const int st = make_plan(p, &pl);
  if (st != COVSPEC_OK) return st;
  if (!workspace || !path_out || ((uintptr_t)workspace & 255u)) return COVSPEC_INVALID_ARG;
  if (pl.lr != COVSPEC_LR_ENERGY_TOPK) return COVSPEC_INVALID_ARG;
  discard_pending_error();
  if (pl.P > 0) {
    HIPCHK(hipMemcpyAsync(path_out, (const char*)workspace + pl.ok, (size_t)pl.B * sizeof(int32_t), hipMemcpyDeviceToDevice,
                          (hipStream_t)stream));
  } else {
    HIPCHK(launch_fill_int(path_out, pl.B, 0, (hipStream_t)stream));
  }
  return COVSPEC_OK;
}

int covspec_image_status(const covspec_params* p, const void* workspace, int32_t* status_out, covspec_stream_t stream) {
  Plan pl;
  const int st = make_plan(p, &pl);
  if (st != COVSPEC_OK) return st;
  if (!workspace || !status_out || ((uintptr_t)workspace & 255u)) return COVSPEC_INVALID_ARG;
  discard_pending_error();
  HIPCHK(hipMemcpyAsync(status_out, (const char*)workspace + pl.status, (size_t)pl.B * sizeof(int32_t), hipMemcpyDeviceToDevice,
                        (hipStream_t)stream));
  return COVSPEC_OK;
}

void covspec_set_wait_limit_us(int64_t microseconds) {
  set_barrier_limit_ticks(microseconds > 0 ? microseconds * 100 : 0);   // 100 ticks of the wall clock per microsecond
}

int covspec_probe_launches(const covspec_params* p, int32_t* rows, int32_t* cols, int32_t* inner) {
  Plan pl;
  if (make_plan(p, &pl) != COVSPEC_OK) return 0;
  if (pl.lr != COVSPEC_LR_ENERGY_TOPK || pl.P <= 0) return 0;
  if (rows) *rows = pl.P;
  if (cols) *cols = pl.nP;
  if (inner) *inner = pl.nP;
  return subspace_product_launches(kSubspaceIters);
}

static int verify_check(const covspec_verify_params* p) {
  if (!p) return COVSPEC_INVALID_ARG;
  if (p->n_seq < 1 || p->n_draft < 1 || p->vocab < 2) return COVSPEC_INVALID_ARG;
  if (p->dtype != COVSPEC_FP32 && p->dtype != COVSPEC_BF16 && p->dtype != COVSPEC_FP16) return COVSPEC_INVALID_ARG;
  // one lane per drafted position in the acceptance kernel (alpha of every position is written in one pass)
  if (p->n_draft > 64 || (long)p->n_seq * p->n_draft > 65535) return COVSPEC_UNSUPPORTED;
  if (p->vocab % (p->dtype == COVSPEC_FP32 ? 4 : 8) != 0) return COVSPEC_UNSUPPORTED;
  return COVSPEC_OK;
}

size_t covspec_verify_workspace_size(const covspec_verify_params* p) {
  if (verify_check(p) != COVSPEC_OK) return 0;
  return verify_workspace_bytes(p->n_seq, p->n_draft, p->vocab, p->dtype);
}

int covspec_verify(const covspec_verify_params* p, const void* z_target, const void* z_draft, const int32_t* tokens,
                   const float* u_accept, const float* u_resample, int32_t* n_accept_out, int32_t* correction_out,
                   float* alpha_out, void* workspace, size_t workspace_bytes, covspec_stream_t stream) {
  const int st = verify_check(p);
  if (st != COVSPEC_OK) return st;
  if (!z_target || !z_draft || !tokens || !u_accept || !u_resample || !n_accept_out || !correction_out || !workspace)
    return COVSPEC_INVALID_ARG;
  if (((uintptr_t)z_target | (uintptr_t)z_draft) & 15) return COVSPEC_INVALID_ARG;
  if ((uintptr_t)workspace & 255) return COVSPEC_INVALID_ARG;
  if (workspace_bytes < verify_workspace_bytes(p->n_seq, p->n_draft, p->vocab, p->dtype)) return COVSPEC_WORKSPACE_TOO_SMALL;
  discard_pending_error();
  const hipError_t e = launch_verify(z_target, z_draft, tokens, u_accept, u_resample, p->n_seq, p->n_draft, p->vocab, p->dtype,
                                     n_accept_out, correction_out, alpha_out, workspace, (hipStream_t)stream);
  if (e != hipSuccess) note_error("launch_verify", e);
  return e == hipSuccess ? COVSPEC_OK : COVSPEC_HIP_ERROR;
}

// ---- covspec_verify for callers that cannot allocate: the per-chunk sums live in a device array of the library.
//
// `scratch` below is, in host code, only a stand-in for the symbol: it is never passed to a kernel or a runtime call.
// Its address on a device comes from hipGetSymbolAddress, looked up once per device with that device current (every
// device holds its own copy of the array at its own address) and kept in g_scratch_ptr.
constexpr size_t kStaticScratchBytes = COVSPEC_VERIFY_STATIC_MAX_SCRATCH;
constexpr int kStaticMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static std::atomic<void*> g_scratch_ptr[kStaticMaxDevices];

// Device address of `scratch` on the current device (nullptr and *err set on failure).
static void* static_scratch_of_current_device(hipError_t* err) {
  int dev = -1;
  if ((*err = hipGetDevice(&dev)) != hipSuccess) return nullptr;
  if (dev < 0 || dev >= kStaticMaxDevices) { *err = hipErrorInvalidDevice; return nullptr; }
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (ptr) return ptr;
  if ((*err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch))) != hipSuccess) return nullptr;
  if (!ptr) { *err = hipErrorInvalidSymbol; return nullptr; }
  g_scratch_ptr[dev].store(ptr, std::memory_order_release);   // two threads racing here store the same address
  return ptr;
}

int covspec_verify_static(const covspec_verify_params* p, const void* z_target, const void* z_draft, const int32_t* tokens,
                          const float* u_accept, const float* u_resample, int32_t* n_accept_out, int32_t* correction_out,
                          float* alpha_out, covspec_stream_t stream) {
  const int st = verify_check(p);
  if (st != COVSPEC_OK) return st;
  if (!z_target || !z_draft || !tokens || !u_accept || !u_resample || !n_accept_out || !correction_out) return COVSPEC_INVALID_ARG;
  if (((uintptr_t)z_target | (uintptr_t)z_draft) & 15) return COVSPEC_INVALID_ARG;
  const size_t need = verify_workspace_bytes(p->n_seq, p->n_draft, p->vocab, p->dtype);
  if (need > kStaticScratchBytes) {
    snprintf(g_last_error, sizeof(g_last_error), "covspec_verify_static: %zu bytes of scratch needed, the static array holds %zu",
             need, kStaticScratchBytes);
    return COVSPEC_UNSUPPORTED;
  }
  discard_pending_error();
  hipError_t e = hipSuccess;
  void* ws = static_scratch_of_current_device(&e);
  if (!ws) {
    note_error("hipGetSymbolAddress of the static scratch array", e);
    return COVSPEC_HIP_ERROR;
  }
  // every partial sum the kernels read was written earlier in the same call, so nothing has to be cleared
  e = launch_verify(z_target, z_draft, tokens, u_accept, u_resample, p->n_seq, p->n_draft, p->vocab, p->dtype, n_accept_out,
                    correction_out, alpha_out, ws, (hipStream_t)stream);
  if (e != hipSuccess) note_error("launch_verify", e);
  return e == hipSuccess ? COVSPEC_OK : COVSPEC_HIP_ERROR;
}

static int draft_check(const covspec_draft_params* p) {
  if (!p) return COVSPEC_INVALID_ARG;
  if (p->n_seq < 1 || p->n_draft < 1 || p->vocab < 2 || p->fanout0 < 0) return COVSPEC_INVALID_ARG;
  if (p->dtype != COVSPEC_FP32 && p->dtype != COVSPEC_BF16 && p->dtype != COVSPEC_FP16) return COVSPEC_INVALID_ARG;
  if (!(p->rho > 0.0 && p->rho < 1.0) || !(p->gamma == p->gamma)) return COVSPEC_INVALID_ARG;   // Sec. III-C: 0 < rho < 1
  if (p->fanout0 > 32 || p->n_draft > 64 || (long)p->n_seq * p->n_draft > 65535) return COVSPEC_UNSUPPORTED;
  if (p->vocab % (p->dtype == COVSPEC_FP32 ? 4 : 8) != 0 || p->vocab > draft_max_vocab()) return COVSPEC_UNSUPPORTED;
  return COVSPEC_OK;
}

int covspec_draft_fanout(const covspec_draft_params* p, int32_t* fanout_out) {
  const int st = draft_check(p);
  if (st != COVSPEC_OK) return st;
  if (!fanout_out) return COVSPEC_INVALID_ARG;
  // F_j = ceil(F_0 rho^j).  rho is a double, so a decimal rho arrives as its nearest double; the product is then
  // off the decimal formula's value by a few 1e-16 relative, which must not tip an exact integer over (F_0 = 30,
  // rho = 0.1: 30 * 0.1 = 3.0000000000000004 in doubles): a product within 1e-12 relative above an integer
  // counts as that integer.
  for (int j = 0; j < p->n_draft; ++j)
    fanout_out[j] = (int32_t)ceil((double)p->fanout0 * pow(p->rho, (double)j) * (1.0 - 1e-12));
  return COVSPEC_OK;
}

size_t covspec_draft_workspace_size(const covspec_draft_params* p) {
  if (draft_check(p) != COVSPEC_OK) return 0;
  return draft_workspace_bytes(p->n_seq, p->n_draft, p->vocab);
}

int covspec_draft_gate(const covspec_draft_params* p, const void* z_draft, const int32_t* tokens, float* margin_out,
                       int32_t* gate_out, int32_t* cand_out, void* workspace, size_t workspace_bytes, covspec_stream_t stream) {
  const int st = draft_check(p);
  if (st != COVSPEC_OK) return st;
  if (!z_draft || !tokens || !margin_out || !gate_out || !workspace || (p->fanout0 > 0 && !cand_out)) return COVSPEC_INVALID_ARG;
  if (((uintptr_t)z_draft & 15) || ((uintptr_t)workspace & 255)) return COVSPEC_INVALID_ARG;
  if (workspace_bytes < draft_workspace_bytes(p->n_seq, p->n_draft, p->vocab)) return COVSPEC_WORKSPACE_TOO_SMALL;
  int32_t fan[64];
  covspec_draft_fanout(p, fan);
  discard_pending_error();
  const hipError_t e = launch_draft(z_draft, tokens, p->n_seq, p->n_draft, p->vocab, p->dtype, p->fanout0, fan, p->gamma, margin_out,
                                    gate_out, cand_out, workspace, (hipStream_t)stream);
  if (e != hipSuccess) note_error("launch_draft", e);
  return e == hipSuccess ? COVSPEC_OK : COVSPEC_HIP_ERROR;
}

const char* covspec_last_error(void) { return g_last_error; }

const char* covspec_status_string(int status) {
  switch (status) {
    case COVSPEC_OK: return "ok";
    case COVSPEC_INVALID_ARG: return "invalid argument";
    case COVSPEC_WORKSPACE_TOO_SMALL: return "workspace too small";
    case COVSPEC_UNSUPPORTED: return "shape or mode outside the kernels' limits";
    case COVSPEC_HIP_ERROR: return "HIP launch error";
    default: return "unknown status";
  }
}

size_t covspec_stream_workspace_size(const covspec_stream_params* p) {
  StreamPlan pl;
  if (make_stream_plan(p, &pl) != COVSPEC_OK) return 0;
  return pl.total;
}

int covspec_stream_step(const covspec_stream_params* p, int32_t n_keep, int32_t id_base, const void* X_frame,
                        const float* s_fused, const void* Z_in, const double* G_in, const int32_t* id_in, void* Z_out,
                        double* G_out, int32_t* id_out, float* c_out, int32_t* n_keep_out, void* workspace,
                        size_t workspace_bytes, covspec_stream_t stream) {
  StreamPlan q;
  int rc = make_stream_plan(p, &q);
  if (rc != COVSPEC_OK) return rc;
  if (n_keep < 0 || n_keep > q.k || !X_frame || !s_fused || !Z_out || !G_out || !id_out) return COVSPEC_INVALID_ARG;
  if (n_keep > 0 && (!Z_in || !G_in || !id_in)) return COVSPEC_INVALID_ARG;
  if (!workspace || ((uintptr_t)workspace & 255u)) return COVSPEC_INVALID_ARG;
  if (workspace_bytes < q.total) return COVSPEC_WORKSPACE_TOO_SMALL;
  hipStream_t st = (hipStream_t)stream;
  void* ws = workspace;
  discard_pending_error();
  const int nC = n_keep + q.M;
  const long d = q.d, gstride = (long)q.nP * q.nP;
  int32_t* idxf = at<int32_t>(ws, q.idxf);
  int32_t* idc = at<int32_t>(ws, q.idc);
  double* Gc = at<double>(ws, q.Gc);

  // 1. the frame's pre-selected tokens and the candidates' ids
  HIPCHK(launch_select_top(s_fused, q.B, q.N, q.M, nullptr, idxf, st));
  HIPCHK(launch_stream_ids(id_in, idxf, idc, q.B, n_keep, q.M, q.k, id_base, st));

  // 2. Gram matrix of the candidates: the kept block is carried, the rows of the arriving tokens are computed
  HIPCHK(launch_fill_zero(Gc, (size_t)q.B * gstride * 8, st));
  HIPCHK(launch_copy_block(Gc, q.nP, gstride, G_in, q.k, (long)q.k * q.k, n_keep, q.B, st));
  GemmArgs g;
  g.A = X_frame; g.lda = d; g.strideA = (long)q.N * d; g.gatherA = idxf; g.gstrideA = q.M;
  g.M = q.M; g.K = q.d; g.ldc = q.nP; g.batch = q.B; g.strideC = gstride;
  g.epilogue = EPI_STORE_F64;
  auto gram = [&](const GemmArgs& a) { return q.dtype == COVSPEC_FP32 ? launch_gemm64_nt(a, false, false, st) : launch_gemm_nt(a, DT_BF16, st); };
  if (n_keep > 0) {
    GemmArgs a = g;            // arriving x kept
    a.B = Z_in; a.ldb = d; a.strideB = (long)q.k * d; a.N = n_keep;
    a.C = Gc + (long)n_keep * q.nP;
    HIPCHK(gram(a));
    HIPCHK(launch_mirror_block(Gc, q.nP, gstride, n_keep, nC, q.B, st));
  }
  {
    GemmArgs a = g;            // arriving x arriving
    a.B = X_frame; a.ldb = d; a.strideB = (long)q.N * d; a.gatherB = idxf; a.gstrideB = q.M; a.N = q.M;
    a.C = Gc + (long)n_keep * q.nP + n_keep;
    HIPCHK(gram(a));
  }

  // 3. keep everything, or the keep_k candidates with the largest energy in the top-r subspace
  const int32_t* sel = nullptr;
  int n_out = nC;
  if (nC > q.k) {
    double* A = at<double>(ws, q.A);
    float* c = c_out ? c_out : at<float>(ws, q.c);
    HIPCHK(hipMemcpyAsync(A, Gc, (size_t)q.B * gstride * 8, hipMemcpyDeviceToDevice, st));   // the solve may overwrite its input
    const int P = subspace_block(nC, q.r);
    if (P > 0) {
      int* ok = at<int>(ws, q.ok);
      const double* Ut = nullptr;
      HIPCHK(launch_subspace_eigen(A, q.B, nC, q.nP, q.r, P, kSubspaceIters, kSubspaceMoreIters, at<void>(ws, q.sub), at<void>(ws, q.ctl),
                                   at<double>(ws, q.lam), ok, &Ut, nullptr, nullptr, nullptr, st));
      HIPCHK(launch_jacobi_eigen(A, q.B, nC, q.nP, q.r, at<void>(ws, q.ctl), at<double>(ws, q.lam), ok, nullptr, nullptr, st));
      HIPCHK(launch_subspace_energy(Ut, q.B, P, nC, q.nP, (long)P * q.nP, q.r, at<double>(ws, q.lam), c, ok, 1, st));
      HIPCHK(launch_subspace_energy(A, q.B, nC, nC, q.nP, gstride, q.r, at<double>(ws, q.lam), c, ok, 0, st));
    } else {
      HIPCHK(launch_jacobi_eigen(A, q.B, nC, q.nP, q.r, at<void>(ws, q.ctl), at<double>(ws, q.lam), nullptr, nullptr, nullptr, st));
      HIPCHK(launch_subspace_energy(A, q.B, nC, nC, q.nP, gstride, q.r, at<double>(ws, q.lam), c, nullptr, 0, st));
    }
    int32_t* selw = at<int32_t>(ws, q.sel);
    HIPCHK(launch_select_top(c, q.B, nC, q.k, nullptr, selw, st));
    sel = selw;
    n_out = q.k;
  }

  // 4. the next state
  HIPCHK(launch_stream_compact(Z_in, X_frame, idxf, sel, idc, Gc, q.nP, gstride, Z_out, id_out, G_out, q.B, n_keep, q.M, q.k, q.N, n_out,
                               (long)q.d * q.esz, st));
  if (n_keep_out) *n_keep_out = n_out;
  return COVSPEC_OK;
}

}  // extern "C"
