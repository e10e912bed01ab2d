/*
 * covspec.h -- C ABI of the MI355X (gfx950) visual-token-reduction library.
 *
 * The library implements the training-free visual token selection of CoVSpec
 * (paper Section III-A, "Visual Token Selection"): score every visual token on
 * query relevance and token activity, fuse the two scores, pre-select the M
 * best, measure each pre-selected token's energy in the top-r singular
 * subspace, keep the B_vis = k tokens with the largest energy and gather their
 * feature rows.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Every data pointer is DEVICE memory owned by the caller.  The library
 *    never allocates or frees memory; scratch space comes from `workspace`.
 *  - All tensors are dense row-major.  B images are independent.
 *  - `dtype` (0 = fp32, 1 = bf16) is the storage type of X, hidden, Q, Wq, Wk
 *    and of the gathered tokens.  Scores are fp32, indices are int32.
 *  - Work is enqueued on `stream`; calls return without synchronising.  Outputs
 *    are valid once the caller has synchronised the stream.
 *  - Arguments are validated on the host before anything is launched.  Return
 *    value: COVSPEC_OK or one of the codes below; no exception crosses the ABI.
 *  - The library keeps no state between calls apart from per-process caches of device properties
 *    (kernel attributes, how many workgroups of a kernel a device holds at once), kept per device and
 *    filled once, and the thread-local text of covspec_last_error(); concurrent calls are safe when
 *    they use distinct workspaces.
 *  - The eigen-solve and the greedy picks of covspec_select / covspec_reduce spread an image over
 *    several workgroups (at most 64) that wait for one another inside one launch, so such a launch
 *    needs that many workgroup slots of the device at the same time.  Alone on the device it always
 *    has them.  Every such wait is bounded (2 s of wall clock unless covspec_set_wait_limit_us says
 *    otherwise): if other work holds the device for longer, the call still ends, COVSPEC_OK has long been
 *    returned, and the image concerned comes back with NaN energies (or NaN residuals) and valid but
 *    meaningless kept indices; covspec_image_status reports which images these are.  Keep concurrent
 *    calls of these two entry points to COVSPEC_MAX_CONCURRENT_CALLS per device.
 *  - Ties in every ranking go to the lower index.  Ranking decisions are taken
 *    on the fp32 score values that the library returns.
 */
#ifndef COVSPEC_H
#define COVSPEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Opaque stream handle: pass a hipStream_t (NULL = the default stream). */
typedef void* covspec_stream_t;

/* Calls of covspec_select / covspec_reduce that may run on one device at the same time without their
 * multi-workgroup kernels starving one another; also the most streams covspec_reduce_ragged takes. */
#define COVSPEC_MAX_CONCURRENT_CALLS 8

enum {
  COVSPEC_OK = 0,
  COVSPEC_INVALID_ARG = 1,         /* NULL required pointer, bad size / mode / lambda ...        */
  COVSPEC_WORKSPACE_TOO_SMALL = 2, /* workspace_bytes < covspec_workspace_size(params)            */
  COVSPEC_UNSUPPORTED = 3,         /* valid request outside the kernels' limits (see below)       */
  COVSPEC_HIP_ERROR = 4            /* a launch failed; covspec_last_error() names the cause       */
};

enum { COVSPEC_FP32 = 0, COVSPEC_BF16 = 1,
       COVSPEC_FP16 = 2 /* logits of covspec_verify and covspec_draft_gate only */ };

/* Query-relevance definition.
 *   COSINE_MAX   : S^query_i = max_j cos(e(v_i), e(q_j))  (paper Sec. III-A.1, query-aware score).
 *   ATTN_SOFTMAX : variant that is NOT in the paper: per head, softmax over the visual tokens of
 *                  e(q_j)_h . e(v_i)_h / sqrt(d/H), averaged over heads and query tokens.        */
enum { COVSPEC_REL_COSINE_MAX = 0, COVSPEC_REL_ATTN_SOFTMAX = 1 };

/* Low-rank stage.
 *   ENERGY_TOPK     : rank-r truncated SVD of the pre-selected tokens, c_i = ||(V_r Sigma_r)_i||^2,
 *                     keep the k largest (paper Sec. III-A.3).
 *   GREEDY_RESIDUAL : variant that is NOT in the paper: k greedy picks, each the token with the
 *                     largest residual after projecting out the tokens already picked
 *                     (pivoted Cholesky of the token Gram matrix).
 * Ablations of the selector (the paper's Table II compares full-token drafting and random-token
 * selection; Sec. III-A.3 names "the M highest-scoring tokens" as the straightforward alternative;
 * full-token drafting is keep_k = preselect_m = n_tokens with any mode):
 *   SCORE_TOPK      : no low-rank term: keep the k highest fused scores.
 *   RANDOM          : keep k tokens drawn uniformly at random, reproducibly: token i of image b gets
 *                     the score (mix64(seed * 0x9E3779B97F4A7C15 + (b << 32 | i) +
 *                     0x632BE59BD9B4E019) >> 40) * 2^-24, mix64 being the output function of the
 *                     SplitMix64 generator, and the k largest are kept (ties -> lower index).
 *                     covspec_reduce then computes no scores at all.                            */
enum { COVSPEC_LR_ENERGY_TOPK = 0, COVSPEC_LR_GREEDY_RESIDUAL = 1, COVSPEC_LR_SCORE_TOPK = 2, COVSPEC_LR_RANDOM = 3 };

typedef struct covspec_params {
  int32_t batch;        /* B >= 1 images                                                          */
  int32_t n_tokens;     /* N visual tokens per image, 1 <= N <= 16384                              */
  int32_t d_model;      /* d feature width; multiple of 8 (bf16) or 4 (fp32)                      */
  int32_t n_query;      /* T >= 1 query-keyword embeddings per image (no padding mask)            */
  int32_t n_heads;      /* H; used by ATTN_SOFTMAX only, which needs (d / H) % 4 == 0            */
  int32_t n_act_layers; /* K in [0, 8]; hidden holds K+1 slices; K = 0 drops the activity term    */
  int32_t dtype;        /* COVSPEC_FP32 / COVSPEC_BF16                                            */
  int32_t rel_mode;     /* COVSPEC_REL_*                                                          */
  int32_t lr_mode;      /* COVSPEC_LR_*                                                           */
  int32_t preselect_m;  /* M; 0 => min(N, 2k).  k <= M <= N, M <= 4096                            */
  int32_t rank_r;       /* r; 0 => max(1, k/2).  1 <= r < min(M, d) (ENERGY_TOPK only)            */
  int32_t keep_k;       /* k; 0 => floor(keep_ratio*N + 0.5) clamped to [1, M]                    */
  float keep_ratio;     /* used only when keep_k == 0; must then be in (0, 1]                     */
  float lambda;         /* fusion weight of the query score, in [0, 1] (paper fusion equation)    */
  uint32_t seed;        /* COVSPEC_LR_RANDOM only                                                 */
} covspec_params;

/* Bytes of device scratch that any of the three entry points needs for `p` (0 if `p` is invalid
 * or unsupported).  The workspace must be 256-byte aligned. */
size_t covspec_workspace_size(const covspec_params* p);

/* Resolve the defaults of `p` (k, M, r) exactly as the entry points do.  Returns a status code. */
int covspec_resolve(const covspec_params* p, int32_t* keep_k, int32_t* preselect_m, int32_t* rank_r);

/*
 * Scores (paper Sec. III-A.1 and III-A.2, fusion equation).
 *   X      [B, N, d]      visual token features (also the representation z_i of the low-rank stage)
 *   hidden [B, K+1, N, d] hidden states of the K+1 last layers, oldest first; NULL (or K = 0) drops
 *                         the activity term and makes s_fused the normalised query score
 *   Q      [B, T, d]      query-keyword features
 *   Wq, Wk [d, d]         embedding maps, [d_in, d_out]: e(q) = q Wq, e(v) = v Wk; NULL = identity
 *   s_query, s_act, s_fused [B, N] fp32 outputs; each may be NULL (s_act is untouched when the
 *                         activity term is dropped)
 * Both scores are min-max normalised per image before fusion; a constant score normalises to 0.
 * A score whose weight in the fusion is zero (lambda = 1: activity, lambda = 0: query relevance, with
 * hidden states given) is computed only when its output pointer is not NULL: 0 * score is an exact
 * zero for finite scores, so s_fused is the same; covspec_reduce passes no score outputs and skips it.
 */
int covspec_score(const covspec_params* p, const void* X, const void* hidden, const void* Q,
                  const void* Wq, const void* Wk, float* s_query, float* s_act, float* s_fused,
                  void* workspace, size_t workspace_bytes, covspec_stream_t stream);

/*
 * Selection from caller-supplied fused scores (paper Sec. III-A.3).
 *   X        [B, N, d]   features; s_fused [B, N] fp32 (RANDOM: ignored, may be NULL)
 *   idx_out  [B, k]      kept token positions in [0, N), ascending              (required)
 *   c_out    [B, M]      ENERGY_TOPK: subspace energy of the pre-selected tokens, in idx_m order;
 *                        other modes: untouched                                  (or NULL)
 *   idx_m_out[B, M]      pre-selected positions, ascending; RANDOM: untouched    (or NULL)
 *   pick_order_out [B,k] GREEDY_RESIDUAL: token positions in pick order          (or NULL)
 *   resid_out [B, k]     GREEDY_RESIDUAL: residual squared norm at each pick     (or NULL)
 */
int covspec_select(const covspec_params* p, const void* X, const float* s_fused, int32_t* idx_out,
                   float* c_out, int32_t* idx_m_out, int32_t* pick_order_out, float* resid_out,
                   void* workspace, size_t workspace_bytes, covspec_stream_t stream);

/*
 * Whole path: score, fuse, select, gather (paper Sec. III-A).
 *   idx_out    [B, k]     kept positions, ascending                              (required)
 *   tokens_out [B, k, d]  bit copies of X[b, idx_out[b, j], :], same dtype as X  (required)
 */
int covspec_reduce(const covspec_params* p, const void* X, const void* hidden, const void* Q,
                   const void* Wq, const void* Wk, int32_t* idx_out, void* tokens_out,
                   void* workspace, size_t workspace_bytes, covspec_stream_t stream);

/*
 * covspec_reduce with per-stage timing marks, for benchmarks and profilers (the paper gives no
 * time breakdown of Sec. III-A; this is how one is measured).  `stage_events` is a HOST array of
 * COVSPEC_NUM_STAGE_EVENTS hipEvent_t handles created by the caller with timing enabled; event i is
 * recorded on `stream` when stage i begins, event COVSPEC_STAGE_END when all work has been enqueued.
 * Stage i lasted from event i to event i+1.  The two probe events bracket ONE launch of the kernel
 * the low-rank stage spends most of its time in (ENERGY_TOPK with the subspace iteration: the fp64
 * product Y^T G of the first iteration, of covspec_probe_launches() equal launches; otherwise they are
 * recorded back to back).  Same results, arguments and errors as covspec_reduce.
 */
enum {
  COVSPEC_STAGE_QUERY_SIDE = 0,       /* weight transposes, e(q) = q Wq, |e(q)|, folded query matrix    */
  COVSPEC_STAGE_TOKEN_PROJECTION = 1, /* x Wk for every token (norms, or e(v) itself for ATTN_SOFTMAX)  */
  COVSPEC_STAGE_RELEVANCE = 2,        /* query/token inner products and the cosine-max / softmax tail    */
  COVSPEC_STAGE_ACTIVITY = 3,         /* activity score stream pass                                      */
  COVSPEC_STAGE_FUSE = 4,             /* min-max normalisation and fusion                                */
  COVSPEC_STAGE_PRESELECT = 5,        /* top-M by fused score                                            */
  COVSPEC_STAGE_GRAM = 6,             /* Gram matrix of the pre-selected tokens                          */
  COVSPEC_STAGE_LOWRANK = 7,          /* eigen-solve (ENERGY_TOPK) or greedy picks (GREEDY_RESIDUAL)     */
  COVSPEC_STAGE_KEEP = 8,             /* subspace energies and top-k, or ordering of the greedy picks    */
  COVSPEC_STAGE_GATHER = 9,           /* gather of the kept rows                                         */
  COVSPEC_STAGE_END = 10,
  COVSPEC_PROBE_BEGIN = 11,
  COVSPEC_PROBE_END = 12,
  COVSPEC_NUM_STAGE_EVENTS = 13
};
int covspec_reduce_staged(const covspec_params* p, const void* X, const void* hidden, const void* Q,
                          const void* Wq, const void* Wk, int32_t* idx_out, void* tokens_out,
                          void* workspace, size_t workspace_bytes, covspec_stream_t stream,
                          void* const* stage_events);

/*
 * Ragged batches: images of different token and keyword counts in one call (not in the paper, whose
 * Sec. III-A treats one image; dynamic-resolution serving batches such images).  Image b of the batch
 * gives exactly the result of covspec_reduce on that image alone, with n_tokens[b] and n_query[b] in
 * place of the template's n_tokens and n_query, k / M / r resolved for that image (from keep_ratio
 * unless the template fixes them), and, for COVSPEC_LR_RANDOM, the draw of image b.
 * `p` is the template: batch, n_tokens and n_query are ignored.  `r` and its arrays are HOST memory.
 * PACKED layouts, image after image, no padding (device pointers):
 *   X          [sum N_b, d];   Q [sum T_b, d];
 *   hidden     image b at element offset (K+1) d sum_{a<b} N_a, shape [K+1, N_b, d]   (or NULL)
 *   idx_out    [sum k_b] int32: positions inside the own image, ascending per image
 *   tokens_out [sum k_b, d]
 * covspec_ragged_resolve writes k_b per image to a host array (output offsets are its prefix sums)
 * and the number of runs.  Consecutive images of equal (N_b, T_b) form a run that is worked off as
 * one dense batch; run i is enqueued on streams[i mod n_streams] with its own slice of the workspace
 * (covspec_ragged_workspace_size bytes for that n_streams, 256-byte aligned).  The caller makes the
 * inputs visible to every stream before the call and synchronises all of them before reading the
 * outputs; with n_streams == 1 the call behaves like the other entry points.  Streams are the
 * caller's (default priority); nothing is created, allocated or synchronised inside.  1 <= n_streams <=
 * COVSPEC_MAX_CONCURRENT_CALLS, else COVSPEC_INVALID_ARG (and a workspace size of 0).  Errors: as
 * covspec_reduce for the first run whose parameters are invalid or unsupported; runs enqueued before
 * a failing one stay enqueued.
 */
typedef struct covspec_ragged {
  int32_t n_images;
  const int32_t* n_tokens;  /* HOST [n_images]: N_b */
  const int32_t* n_query;   /* HOST [n_images]: T_b */
} covspec_ragged;

int covspec_ragged_resolve(const covspec_params* p, const covspec_ragged* r, int32_t* keep_k_out,
                           int32_t* n_runs_out);
size_t covspec_ragged_workspace_size(const covspec_params* p, const covspec_ragged* r, int32_t n_streams);
int covspec_reduce_ragged(const covspec_params* p, const covspec_ragged* r, const void* X,
                          const void* hidden, const void* Q, const void* Wq, const void* Wk,
                          int32_t* idx_out, void* tokens_out, void* workspace, size_t workspace_bytes,
                          const covspec_stream_t* streams, int32_t n_streams);

/*
 * covspec_stream_step: the frame-by-frame form of the low-rank selection for video whose frames arrive one by
 * one.  NOT in the paper, which selects the tokens of one image at once (Sec. III-A.3); defined so that every
 * frame is exactly one application of that section (stack the candidates, rank-r SVD, energy, keep the
 * largest) to the candidate set "tokens kept so far, then the frame's pre-selected tokens":
 *   1. the frame_m tokens of the frame with the largest s_fused are pre-selected (ascending position);
 *   2. candidates = the n_keep kept tokens in their order, then the pre-selected ones: n_C = n_keep + frame_m;
 *   3. n_C <= keep_k: every candidate is kept.  Otherwise c_i = energy of candidate i in the top-r singular
 *      subspace of the n_C candidate rows, and the keep_k candidates with the largest c (fp32 values, ties to
 *      the earlier candidate) are kept, in candidate order.
 * The kept tokens' Gram matrix travels with the state, so only the frame_m rows of the arriving tokens are
 * computed (frame_m * n_C * d products instead of n_C^2 * d); the kept block is copied and, after the
 * decision, gathered.  `batch` independent videos advance together, one frame each, all with the same n_keep.
 * State, owned by the caller, device memory, one set read and another written (they must not overlap; swap
 * them between frames; before the first frame n_keep = 0 and the input set is not read):
 *   Z  [batch, keep_k, d] feature rows in the storage dtype;  G [batch, keep_k, keep_k] fp64, G_ij = z_i . z_j;
 *   id [batch, keep_k] int32 caller-side token ids (an arriving token gets id_base + its position in the
 *   frame).  Rows and entries at or beyond the kept count are unspecified.
 * X_frame [batch, n_frame, d], s_fused [batch, n_frame] fp32 (covspec_score of the frame, or any score).
 * c_out (optional) [batch, n_keep + frame_m] fp32 energies, written only when n_C > keep_k.
 * *n_keep_out (HOST, optional) = min(keep_k, n_keep + frame_m), the count to pass with the next frame.
 * Precision as covspec_select: bf16 storage takes the Gram rows on the bf16 MFMA with fp32 partial sums flushed
 * into fp64, fp32 storage on the fp64 MFMA; the eigen-solve is fp64.
 * Errors: COVSPEC_INVALID_ARG (NULL pointer, n_keep outside 0..keep_k, frame_m outside 1..n_frame, rank_r
 * outside 1..min(keep_k, d_model)-1, misaligned workspace), COVSPEC_UNSUPPORTED (keep_k + frame_m > 4096,
 * n_frame > 16384, d_model not a multiple of 8 (bf16) / 4 (fp32)), COVSPEC_WORKSPACE_TOO_SMALL, COVSPEC_HIP_ERROR.
 */
typedef struct covspec_stream_params {
  int32_t batch;     /* videos advancing together                     */
  int32_t n_frame;   /* N_f: tokens per arriving frame                 */
  int32_t d_model;
  int32_t dtype;     /* COVSPEC_FP32 / COVSPEC_BF16: X_frame and Z     */
  int32_t frame_m;   /* M_f: pre-selected per frame                    */
  int32_t keep_k;    /* k: tokens kept across frames                   */
  int32_t rank_r;    /* r                                              */
} covspec_stream_params;

size_t covspec_stream_workspace_size(const covspec_stream_params* p);
int covspec_stream_step(const covspec_stream_params* p, int32_t n_keep, int32_t id_base, const void* X_frame,
                        const float* s_fused, const void* Z_in, const double* G_in, const int32_t* id_in,
                        void* Z_out, double* G_out, int32_t* id_out, float* c_out, int32_t* n_keep_out,
                        void* workspace, size_t workspace_bytes, covspec_stream_t stream);

/*
 * Which way each image's eigen-solve went in the LAST covspec_select / covspec_reduce call with these
 * parameters on this workspace (COVSPEC_LR_ENERGY_TOPK only; diagnostics for tests and tuning: the
 * paper's Sec. III-A.3 asks for a rank-r SVD and says nothing of how).  path_out: DEVICE int32 [B]:
 *   1  block subspace iteration, converged at the first residual check
 *   2  converged after the additional steps of the second pass
 *   0  full Jacobi solve of the Gram matrix (fallback, or the block would be most of the matrix)
 * Enqueued on `stream` after the call in question; reads the workspace, writes nothing else.
 */
int covspec_lowrank_path(const covspec_params* p, const void* workspace, int32_t* path_out,
                         covspec_stream_t stream);

/*
 * Per-image outcome of the LAST covspec_select / covspec_reduce call with these parameters on this workspace:
 * status_out (DEVICE int32 [B]) is 0 for an image whose result is valid and 1 for an image whose eigen-solve or
 * greedy picks gave up because a workgroup waited for the others of its image beyond the wait limit (the device
 * was held by other work).  For such an image the kept indices and gathered tokens are meaningless (energies and
 * residuals are NaN) and the call should be repeated.  The status word is cleared at the start of every call and
 * only ever set by the kernels that wait; modes without such kernels (SCORE_TOPK, RANDOM) always report 0.
 * Enqueued on `stream` behind the call in question; reads the workspace, writes nothing else.  (The selection
 * method itself, paper Sec. III-A.3, has no failure case: this reports a property of the execution.)
 * covspec_reduce_ragged keeps one status word per run inside its workspace slices and has no such query.
 */
int covspec_image_status(const covspec_params* p, const void* workspace, int32_t* status_out,
                         covspec_stream_t stream);

/*
 * Wait limit of the multi-workgroup kernels (see the conventions above), process-wide, in microseconds of wall
 * clock; read when a call is enqueued.  Values <= 0 restore the default of 2 000 000.  A limit shorter than a
 * workgroup's normal wait (tens of microseconds) makes images give up spuriously: tests of the give-up path use
 * that, every kernel still runs to its end.
 */
void covspec_set_wait_limit_us(int64_t microseconds);

/*
 * Description of the probed launch for these parameters: number of equal launches per call (0 when
 * nothing is probed) and, if non-NULL, its dimensions: the product is [rows x inner] * [inner x cols]
 * per image in fp64 (2*rows*cols*inner flops per image).
 */
int covspec_probe_launches(const covspec_params* p, int32_t* rows, int32_t* cols, int32_t* inner);

/*
 * Speculative verification over the vocabulary (paper Sec. II-A: the softmax distributions of the
 * draft and the target model, the acceptance probability of a drafted token, and the residual
 * distribution a correction is drawn from after the first rejection).  For each of n_seq sequences
 * with n_draft drafted positions tau = 0..n_draft-1 and vocabulary width vocab:
 *   p_t = softmax(z_target[s, tau, :]), p_d = softmax(z_draft[s, tau, :]);
 *   alpha[s, tau] = min(1, p_t(y) / p_d(y)) at the drafted token y = tokens[s, tau];
 *   position tau is accepted iff u_accept[s, tau] < alpha[s, tau] (both fp32);
 *   n_accept[s] = number of accepted positions before the first rejection;
 *   if n_accept[s] < n_draft: correction[s] = the smallest word w whose cumulative residual mass
 *   sum_{v <= w} max(p_t(v) - p_d(v), 0) at tau = n_accept[s] exceeds u_resample[s] times the total
 *   (inverse CDF in vocabulary order; argmax p_t, lowest index, if the total is zero);
 *   otherwise correction[s] = -1 (the bonus token needs target logits of one more position).
 * The random numbers are inputs: uniforms in [0, 1) drawn by the caller.
 *
 * All pointers are DEVICE pointers, dense row-major, 16-byte aligned:
 *   z_target, z_draft [n_seq, n_draft, vocab]  dtype (fp32, or bf16 / fp16 bit patterns)
 *   tokens            [n_seq, n_draft] int32 in [0, vocab); a value outside is clamped into the range
 *   u_accept          [n_seq, n_draft] fp32;  u_resample [n_seq] fp32
 *   n_accept_out      [n_seq] int32 (required);  correction_out [n_seq] int32 (required)
 *   alpha_out         [n_seq, n_draft] fp32 (or NULL)
 * Limits: vocab a multiple of 8 (bf16, fp16) or 4 (fp32), 2 <= vocab, n_draft <= 64, n_seq * n_draft <= 65535,
 * else COVSPEC_UNSUPPORTED.  The workspace (covspec_verify_workspace_size bytes, 256-byte aligned, owned
 * by the caller, contents undefined between calls) holds per-chunk partial sums.  Work is enqueued on
 * `stream`; the call does not synchronise and allocates nothing.  Returns a covspec_status.
 */
typedef struct covspec_verify_params {
  int32_t n_seq;    /* S: sequences verified in one call                    */
  int32_t n_draft;  /* L: drafted positions per sequence                    */
  int32_t vocab;    /* V: vocabulary width                                  */
  int32_t dtype;    /* covspec_dtype of the logits                          */
} covspec_verify_params;

/* Bytes of workspace covspec_verify needs (0 if the parameters are invalid or unsupported). */
size_t covspec_verify_workspace_size(const covspec_verify_params* p);

int covspec_verify(const covspec_verify_params* p, const void* z_target, const void* z_draft,
                   const int32_t* tokens, const float* u_accept, const float* u_resample,
                   int32_t* n_accept_out, int32_t* correction_out, float* alpha_out,
                   void* workspace, size_t workspace_bytes, covspec_stream_t stream);

/*
 * covspec_verify for callers that cannot allocate device memory or have no workspace to hand over: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and errors
 * as covspec_verify without the workspace: the per-chunk sums go to a device array that is part of the library
 * (COVSPEC_VERIFY_STATIC_MAX_SCRATCH bytes on every device the library runs on, held until the process ends).
 * The call allocates and frees nothing and synchronises nothing; the array's address is looked up on the first
 * call on a device.  Shapes whose workspace (covspec_verify_workspace_size) exceeds the array are refused with
 * COVSPEC_UNSUPPORTED before anything is launched (covspec_last_error() then names both sizes).  All calls on one
 * device share the array: two calls that may overlap on a device (different streams, or threads) race on it and
 * give undefined results; calls on one stream are ordered and safe.  Nothing in the array needs clearing between
 * calls: every value a call reads it has written itself.
 */
#define COVSPEC_VERIFY_STATIC_MAX_SCRATCH (1u << 20)
int covspec_verify_static(const covspec_verify_params* p, const void* z_target, const void* z_draft,
                          const int32_t* tokens, const float* u_accept, const float* u_resample,
                          int32_t* n_accept_out, int32_t* correction_out, float* alpha_out,
                          covspec_stream_t stream);

/*
 * Draft-side vocabulary pass: margin gate (paper Sec. III-B, the margin and gating equations) and
 * bonus-token candidates for parallel branching (Sec. III-C, the fan-out equation and the candidate
 * rule), from one read of the draft logits.  For each of n_seq sequences and each position
 * j = 0..n_draft-1 of its drafted segment, with p_d = softmax(z_draft[s, j, :]):
 *   margin[s, j] = p_(1) - p_(2), the two largest probabilities;
 *   gate[s, j]   = 0 if margin >= gamma (commit locally), 1 otherwise (verify); compared in fp32;
 *   F_j          = ceil(fanout0 * rho^j), evaluated on the host in double precision (a product within 1e-12
 *                  relative above an integer counts as that integer, so that a decimal rho gives the value of
 *                  the decimal formula: fanout0 = 30, rho = 0.1 gives F_1 = 3);
 *   cand[s, j, 0..F_j-1] = the F_j words with the largest draft logits other than tokens[s, j], by
 *                  descending logit, the lower word first among equal logits; entries from F_j (or from
 *                  vocab - 1, if smaller) up to fanout0 are -1.
 * covspec_draft_fanout writes F_0..F_{n_draft-1} to a HOST array.  Other pointers are DEVICE pointers,
 * dense row-major, z_draft 16-byte aligned:
 *   z_draft [n_seq, n_draft, vocab] dtype;  tokens [n_seq, n_draft] int32 (a value outside [0, vocab)
 *   excludes nothing);  margin_out [n_seq, n_draft] fp32 (required);  gate_out [n_seq, n_draft] int32
 *   (required);  cand_out [n_seq, n_draft, fanout0] int32 (required unless fanout0 == 0).
 * Limits: 0 <= fanout0 <= 32, 0 < rho < 1, n_draft <= 64, n_seq * n_draft <= 65535, vocab a multiple of
 * 8 (bf16, fp16) or 4 (fp32) and at most 524288, else COVSPEC_INVALID_ARG / COVSPEC_UNSUPPORTED.  Workspace as
 * for covspec_verify (covspec_draft_workspace_size bytes, 256-byte aligned).  Enqueues on `stream`,
 * does not synchronise, allocates nothing.  Returns a covspec_status.
 */
typedef struct covspec_draft_params {
  int32_t n_seq;    /* S                                                    */
  int32_t n_draft;  /* L: positions per drafted segment                     */
  int32_t vocab;    /* V                                                    */
  int32_t dtype;    /* covspec_dtype of the logits                          */
  int32_t fanout0;  /* F_0: candidates at the first position                */
  double rho;       /* decay of the fan-out, 0 < rho < 1                    */
  float gamma;      /* margin threshold of the gate                         */
} covspec_draft_params;

int covspec_draft_fanout(const covspec_draft_params* p, int32_t* fanout_out);
size_t covspec_draft_workspace_size(const covspec_draft_params* p);
int covspec_draft_gate(const covspec_draft_params* p, const void* z_draft, const int32_t* tokens,
                       float* margin_out, int32_t* gate_out, int32_t* cand_out,
                       void* workspace, size_t workspace_bytes, covspec_stream_t stream);

/* Static, NUL-terminated description of a status code. */
const char* covspec_status_string(int status);

/* After a COVSPEC_HIP_ERROR on this host thread: the HIP error name and the launch step that
 * reported it (NUL-terminated, thread-local, valid until the thread's next failing call; empty if
 * none).  An entry point discards any error an earlier runtime call of the thread left pending
 * before its first launch, so what is reported belongs to the call that returned the status. */
const char* covspec_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* COVSPEC_H */
