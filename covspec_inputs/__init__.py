"""Seeded synthetic inputs for the visual-token-reduction path.

This module only *draws* inputs (visual features, late-layer hidden states,
query-keyword embeddings, projection weights) and converts storage formats.
It contains none of the method's arithmetic (no scores, no selection), so both
the CPU oracle's tests and the HIP path's tests can consume the same arrays
without sharing any implementation.

The paper evaluates on VQAv2 / MMMU / MMBench features of InternVL2.5
(Section IV, experimental setup); none of those are available offline, so the
five workloads below stand in for them: they reproduce token counts, widths,
keep ratios and the structure each score reacts to (low-rank factors,
duplicates, norm outliers, temporal drift).

Conventions
-----------
* ``N(0, x)`` for weights means variance ``x`` (std ``x**0.5``); for additive
  noise / drift the number is a standard deviation relative to unit-RMS signal.
* Every array is produced in float32 and rounded once (round-to-nearest-even)
  to the storage dtype.  bf16 arrays are returned as ``uint16`` bit patterns.
* Seeds: image ``b`` of config ``c`` uses ``BASE_SEED + 1000*c + b``; the
  weights of config ``c`` use ``BASE_SEED + 1000*c + 999``.  Streams are drawn
  in the fixed order U, W, noise, structure, Q, hidden.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

BASE_SEED = 260502218

FP32 = 0
BF16 = 1
FP16 = 2      # logits of the vocabulary passes only; stored as uint16 bit patterns like bf16


@dataclass(frozen=True)
class Workload:
    """Shape and structure of one synthetic workload."""

    cid: int
    name: str
    batch: int          # B images
    n_tokens: int       # N visual tokens per image
    d_model: int        # d feature width
    dtype: int          # FP32 or BF16 storage
    n_query: int        # T query-keyword embeddings per image
    n_heads: int        # H (only the attention-softmax relevance variant uses it)
    keep_k: int         # k = B_vis kept tokens
    preselect_m: int    # M pre-selected tokens
    rank_r: int         # r retained rank
    factor_rank: int    # R of the generating factor
    n_act_layers: int = 4   # K late layers (hidden holds K+1 slices)
    lam: float = 0.5        # lambda of the score fusion
    structure: str = "plain"
    noise_std: float = 0.01


WORKLOADS: Dict[int, Workload] = {
    1: Workload(1, "tiny-fp32", 1, 576, 1024, FP32, 16, 8, 64, 128, 32, 64),
    2: Workload(2, "llava15-like", 1, 576, 4096, BF16, 32, 32, 144, 288, 72, 256,
                structure="dups+outliers"),
    3: Workload(3, "qwen2vl-like", 8, 2304, 3584, BF16, 64, 28, 576, 1152, 288, 384,
                structure="blobs"),
    4: Workload(4, "video-8x1024", 4, 8192, 1536, BF16, 64, 12, 819, 1638, 128, 256,
                structure="video"),
    5: Workload(5, "anyres-batch64", 64, 2880, 4096, BF16, 128, 32, 320, 640, 160, 512,
                structure="neardups"),
}


# --------------------------------------------------------------------------
# storage-format helpers
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def store(x: np.ndarray, dtype: int) -> np.ndarray:
    """Round a float32 array once to the storage dtype."""
    if dtype == FP32:
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == FP16:
        return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)
    return f32_to_bf16_bits(x)


def as_f32(a: np.ndarray, dtype: int) -> np.ndarray:
    """Stored array -> float32 with exactly the stored values."""
    if dtype == FP32:
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == FP16:
        return np.ascontiguousarray(a, dtype=np.uint16).view(np.float16).astype(np.float32)
    return bf16_bits_to_f32(a)


def as_f64(a: np.ndarray, dtype: int) -> np.ndarray:
    """Stored array -> float64 with exactly the stored values."""
    return as_f32(a, dtype).astype(np.float64)


# --------------------------------------------------------------------------
# generators
# --------------------------------------------------------------------------
def _randn(rng: np.random.Generator, *shape: int) -> np.ndarray:
    return rng.standard_normal(shape, dtype=np.float32)


def _factor(rng, n, d, R, u_rows: Optional[np.ndarray] = None) -> np.ndarray:
    """Unit-RMS rank-R factor U diag(S) W with S geometric 1 -> 0.01."""
    U = _randn(rng, n, R) if u_rows is None else u_rows
    W = _randn(rng, R, d)
    S = (0.01 ** (np.arange(R, dtype=np.float64) / max(R - 1, 1))).astype(np.float32)
    scale = np.float32(1.0 / np.sqrt(np.sum(S.astype(np.float64) ** 2)))
    return (U * (S * scale)[None, :]) @ W


def make_image(w: Workload, b: int, seed: Optional[int] = None) -> Dict[str, np.ndarray]:
    """One image's inputs: X [N,d], Q [T,d], hidden [K+1,N,d] in storage dtype."""
    rng = np.random.default_rng(np.random.PCG64(BASE_SEED + 1000 * w.cid + b if seed is None else seed))
    N, d, R = w.n_tokens, w.d_model, w.factor_rank
    dup_dst = dup_src = None

    if w.structure == "blobs":
        centres = _randn(rng, 48, R)
        which = rng.integers(0, 48, size=N)
        U = centres[which] + np.float32(0.3) * _randn(rng, N, R)
        X = _factor(rng, N, d, R, U)
        X += np.float32(w.noise_std) * _randn(rng, N, d)
    elif w.structure == "video":
        per = 1024
        frames = N // per
        X = np.empty((N, d), dtype=np.float32)
        X[:per] = _factor(rng, per, d, R)
        X[:per] += np.float32(w.noise_std) * _randn(rng, per, d)
        for f in range(1, frames):
            X[f * per:(f + 1) * per] = X[(f - 1) * per:f * per] + np.float32(0.05) * _randn(rng, per, d)
        if N > frames * per:  # ragged tail for custom sizes
            X[frames * per:] = _factor(rng, N - frames * per, d, R)
    else:
        X = _factor(rng, N, d, R)
        X += np.float32(w.noise_std) * _randn(rng, N, d)

    if w.structure == "dups+outliers":
        n_dup = max(1, round(0.05 * N))
        perm = rng.permutation(N)
        dup_dst, dup_src, outl = perm[:n_dup], perm[n_dup:2 * n_dup], perm[2 * n_dup:2 * n_dup + 8]
        X[dup_dst] = X[dup_src]
        X[outl] *= np.float32(20.0)
    elif w.structure == "neardups":
        n_dup = N // 10
        perm = rng.permutation(N)
        dst, src = perm[:n_dup], perm[n_dup:2 * n_dup]
        X[dst] = X[src] + np.float32(1e-3) * _randn(rng, n_dup, d)

    Q = _randn(rng, w.n_query, d)

    K = w.n_act_layers
    Xs = store(X, w.dtype)
    hidden = np.empty((K + 1,) + Xs.shape, dtype=Xs.dtype)
    hidden[0] = Xs
    a = np.exp(rng.normal(-1.0, 0.75, size=N)).astype(np.float32)
    prev = as_f32(Xs, w.dtype)
    inv_sqrt_d = np.float32(1.0 / np.sqrt(d))
    for l in range(1, K + 1):
        prev = prev + (a * inv_sqrt_d)[:, None] * _randn(rng, N, d)
        hidden[l] = store(prev, w.dtype)
        prev = as_f32(hidden[l], w.dtype)
    if dup_dst is not None:
        hidden[:, dup_dst] = hidden[:, dup_src]

    return {"X": Xs, "Q": store(Q, w.dtype), "hidden": hidden}


def make_weights(w: Workload, seed: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Projection weights Wq, Wk: [d_in, d_out], entries N(0, 1/d)."""
    rng = np.random.default_rng(np.random.PCG64(BASE_SEED + 1000 * w.cid + 999 if seed is None else seed))
    d = w.d_model
    s = np.float32(1.0 / np.sqrt(d))
    Wq = store(s * _randn(rng, d, d), w.dtype)
    Wk = store(s * _randn(rng, d, d), w.dtype)
    return {"Wq": Wq, "Wk": Wk}


def make_batch(w: Workload, images=None) -> Dict[str, np.ndarray]:
    """Stack the inputs of ``images`` (default: all B) plus the shared weights."""
    images = list(range(w.batch)) if images is None else list(images)
    per = [make_image(w, b) for b in images]
    out = {k: np.stack([p[k] for p in per]) for k in ("X", "Q", "hidden")}
    out.update(make_weights(w))
    return out


def small_workload(cid: int = 0, **kw) -> Workload:
    """A custom (test-sized) workload; unspecified fields come from config 1."""
    return replace(WORKLOADS[1], cid=cid, name=kw.pop("name", "custom"), **kw)


def make_spectrum_tokens(n: int, d: int, sigma: np.ndarray, seed: int, dtype: int = FP32) -> np.ndarray:
    """n tokens of width d >= n whose singular values are exactly ``sigma`` (before the one rounding to the
    storage dtype): X = U diag(sigma) W^T with U (n x n) and W (d x n) the orthonormal factors of Gaussian
    matrices.  For tests that need a prescribed decay of the Gram matrix's eigenvalues sigma^2."""
    rng = np.random.default_rng(BASE_SEED + 700000 + seed)
    U, _ = np.linalg.qr(rng.standard_normal((n, n)))
    W, _ = np.linalg.qr(rng.standard_normal((d, n)))
    X = (U * np.asarray(sigma, dtype=np.float64)[None, :]) @ W.T
    return store(X.astype(np.float32), dtype)


def make_video_stream(n_frames: int, n_frame: int, d: int, dtype: int = BF16, seed: int = 0, factor_rank: int = 64,
                      noise_std: float = 0.05, drift: float = 0.25, cut_every: int = 0):
    """One video as frames that arrive one by one: X [n_frames, n_frame, d] in the storage dtype and fused
    scores s [n_frames, n_frame] (float32, uniform in [0, 1): what a score pass over the frame would hand on).
    Frame 0 is the low-rank-plus-noise token model of the image workloads; frame f is frame f-1 with every token
    moved by `drift` times a fresh draw of the same model (slowly changing content, as in workload 4), and, when
    cut_every > 0, a fresh scene every cut_every frames."""
    rng = np.random.default_rng(BASE_SEED + 800000 + seed)
    R = min(factor_rank, d, n_frame)
    X = np.empty((n_frames, n_frame, d), dtype=np.float32)
    def fresh():
        return _factor(rng, n_frame, d, R) + np.float32(noise_std) * _randn(rng, n_frame, d)
    X[0] = fresh()
    for f in range(1, n_frames):
        X[f] = fresh() if (cut_every and f % cut_every == 0) else X[f - 1] + np.float32(drift) * fresh()
    s = rng.random((n_frames, n_frame), dtype=np.float32)
    return store(X, dtype), s


# --------------------------------------------------------------------------
# logits for the speculative verification step (paper Sec. II-A)
# --------------------------------------------------------------------------
VERIFY_VOCAB = 151936      # vocabulary width of the stand-in workload (a current open LLM tokenizer's, padded)


def make_verify_batch(n_seq: int, n_draft: int, vocab: int, dtype: int = BF16, seed: int = 0,
                      disagreement: float = 0.6, peak: Optional[float] = None, copy_rows: int = 0) -> Dict[str, np.ndarray]:
    """Draft/target logits, drafted tokens and uniforms for ``n_seq`` sequences of ``n_draft`` positions.

    The paper measures on the logits of InternVL2.5 models; these stand in for them with the structure the
    verification step reacts to.  Target logits are N(0, 2^2) over the vocabulary with a handful of boosted
    words per row (+``peak`` on one word, +``peak``/2 on three more), so that each row's distribution is peaked
    like a language model's.  With ``peak=None`` every row draws its own boost, ln(V) + 2 + N(0, 2^2): the top
    word then holds anything from a few percent to nearly all of the mass (the N(0, 2^2) body of V words weighs
    about V e^2), so confident and uncertain positions both occur.  Draft logits are the target's plus N(0, ``disagreement``^2) noise, so that the two
    models mostly agree.  In the first ``copy_rows`` sequences the draft row equals the target row exactly
    (acceptance probability one, empty residual).  The drafted token is a draw from the draft's distribution,
    taken as the argmax of draft logits plus Gumbel noise, which needs no normalisation.  Uniforms are float32
    in [0, 1).  Logits are rounded once to the storage dtype BEFORE the drafted token is drawn.
    Streams are drawn in the fixed order target, boosted words, boosts, noise, Gumbel, uniforms.
    """
    rng = np.random.default_rng(BASE_SEED + 500000 + seed)
    S, L, V = n_seq, n_draft, vocab
    zt = 2.0 * rng.standard_normal((S, L, V), dtype=np.float32)
    hot = rng.integers(0, V, size=(S, L, 4))
    if peak is None:
        boost = (np.log(V) + 2.0 + 2.0 * rng.standard_normal((S, L, 1))).astype(np.float32)
    else:
        boost = np.full((S, L, 1), peak, dtype=np.float32)
    for j in range(4):
        np.put_along_axis(zt, hot[:, :, j:j + 1], (boost if j == 0 else boost / 2) +
                          np.take_along_axis(zt, hot[:, :, j:j + 1], axis=2), axis=2)
    zd = zt + np.float32(disagreement) * rng.standard_normal((S, L, V), dtype=np.float32)
    zd[:copy_rows] = zt[:copy_rows]
    zt_s, zd_s = store(zt, dtype), store(zd, dtype)
    g = rng.gumbel(size=(S, L, V)).astype(np.float32)
    tok = np.argmax(as_f32(zd_s, dtype) + g, axis=2).astype(np.int32)
    u_acc = rng.random((S, L), dtype=np.float32)
    u_res = rng.random(S, dtype=np.float32)
    return {"zt": zt_s, "zd": zd_s, "tok": tok, "u_acc": u_acc, "u_res": u_res}
