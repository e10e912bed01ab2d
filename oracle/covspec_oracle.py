"""CPU oracle for CoVSpec's training-free visual token selection.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
path computes, written from the paper (Section III-A, "Visual Token
Selection").  It is imported only by tests, by the smoke check and by the
benchmark's reported CPU baseline; the product path never calls it and shares
no code with it.  Everything is float64 NumPy; library primitives used as
steps: matmul, SVD, stable sort.

Steps, in the paper's order (per image; images are independent):

1. embeddings e(v_i) = x_i W_k, e(q_j) = q_j W_q            (Sec. III-A.1; the
   paper leaves e(.) open, the workloads supply linear maps; None = identity)
2. query-aware score  S^query_i = max_j cos(e(v_i), e(q_j))   (query-aware score eq.)
   variant "attn": per-head softmax over visual tokens of scaled dot products,
   averaged over heads and query tokens (NOT in the paper; kept as a named
   variant because the build target lists it)
3. activity score     S^act_i = (1/K) sum_l ||h_i^(l) - h_i^(l-1)||_2   (activity eq.)
4. per-image min-max normalisation of both, fused score
   S_i = lam*S^query_i + (1-lam)*S^act_i                      (fusion eq.)
5. pre-select the M tokens with the largest S                  (Sec. III-A.3)
6. Z_M = their feature vectors; truncated SVD of rank r;
   c_i = || (V_r Sigma_r)_{i,:} ||^2                          (stacking / SVD / energy eqs.)
7. keep the B_vis = k tokens with the largest c_i              (end of Sec. III-A.3)
   variant "greedy": pivoted-Cholesky / column-pivoted Gram-Schmidt picks
   (NOT in the paper; named variant)
   ablations of the selector (Table II compares full-token drafting and random-token
   selection; Sec. III-A.3 names top-M by score as the straightforward alternative):
   "score": keep the k highest fused scores; "random": keep k tokens drawn uniformly at
   random from a counter-based generator that the GPU path implements too
8. gather the kept feature rows.

Readings where the paper is silent (all listed in the design notes):
zero-norm vectors score 0 (denominator floored at 1e-30); "normalise to the
same scale" = per-image min-max, constant vector -> zeros; ties everywhere go
to the lower index; kept indices are returned ascending; every ranking
decision is taken on the score rounded to float32, the precision in which the
library returns scores (so the GPU path and this oracle decide in the same
precision).

Parity status: every function below is pinned by tests/test_oracle_pins.py
(closed forms, invariants, brute force, textbook special cases).  Unpinned by
construction: the *choice* of lam, K, M, r and of min-max normalisation, and
the downstream accuracy effect reported in the paper's ablation table (needs
datasets and models that are not available): parity unpinned for those.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np

REL_COSINE_MAX = 0
REL_ATTN_SOFTMAX = 1
LR_ENERGY_TOPK = 0
LR_GREEDY_RESIDUAL = 1
LR_SCORE_TOPK = 2      # ablation: keep the k highest fused scores, no low-rank term (Sec. III-A.3, first sentence)
LR_RANDOM = 3          # ablation: k tokens drawn uniformly at random (the "random-token selection" row of Table II)


@dataclass
class Params:
    n_heads: int = 1
    rel_mode: int = REL_COSINE_MAX
    lr_mode: int = LR_ENERGY_TOPK
    preselect_m: int = 0
    rank_r: int = 0
    keep_k: int = 0
    keep_ratio: float = 0.25
    lam: float = 0.5
    seed: int = 0

    def resolved(self, n_tokens: int):
        """(k, M, r) after applying the defaults of the C interface."""
        k = self.keep_k if self.keep_k > 0 else int(np.floor(self.keep_ratio * n_tokens + 0.5))
        M = self.preselect_m if self.preselect_m > 0 else min(n_tokens, 2 * k)
        k = max(1, min(k, M))
        r = self.rank_r if self.rank_r > 0 else max(1, k // 2)
        return k, M, r


# --------------------------------------------------------------------------
# step 1: embeddings
# --------------------------------------------------------------------------
def embed(A: np.ndarray, W: Optional[np.ndarray]) -> np.ndarray:
    """e(a) = a W for row vectors a; W is [d_in, d_out]; None means identity."""
    A = np.asarray(A, dtype=np.float64)
    return A if W is None else A @ np.asarray(W, dtype=np.float64)


# --------------------------------------------------------------------------
# step 2: query relevance
# --------------------------------------------------------------------------
def cosine_matrix(Ev: np.ndarray, Eq: np.ndarray) -> np.ndarray:
    """cos[i, j] = <Ev_i, Eq_j> / (||Ev_i|| ||Eq_j||), denominator floored at 1e-30."""
    nv = np.sqrt(np.sum(Ev * Ev, axis=1))
    nq = np.sqrt(np.sum(Eq * Eq, axis=1))
    return (Ev @ Eq.T) / np.maximum(nv[:, None] * nq[None, :], 1e-30)


def query_score_cosine(Ev: np.ndarray, Eq: np.ndarray) -> np.ndarray:
    """Query-aware score: maximum cosine similarity over the query keywords."""
    return cosine_matrix(Ev, Eq).max(axis=1)


def attention_rows(Ev: np.ndarray, Eq: np.ndarray, n_heads: int) -> np.ndarray:
    """A[h, j, :] = softmax over visual tokens i of Eq[j,h] . Ev[i,h] / sqrt(dh)."""
    N, d = Ev.shape
    T = Eq.shape[0]
    dh = d // n_heads
    A = np.empty((n_heads, T, N), dtype=np.float64)
    for h in range(n_heads):
        cols = slice(h * dh, (h + 1) * dh)
        logits = (Eq[:, cols] @ Ev[:, cols].T) / np.sqrt(dh)
        logits = logits - logits.max(axis=1, keepdims=True)
        e = np.exp(logits)
        A[h] = e / e.sum(axis=1, keepdims=True)
    return A


def query_score_attention(Ev: np.ndarray, Eq: np.ndarray, n_heads: int) -> np.ndarray:
    """Variant relevance: attention mass a token receives, averaged over heads and queries."""
    return attention_rows(Ev, Eq, n_heads).mean(axis=(0, 1))


# --------------------------------------------------------------------------
# step 3: token activity
# --------------------------------------------------------------------------
def activity_score(Hs: np.ndarray) -> np.ndarray:
    """Hs is [K+1, N, d], slice l-1 -> l are consecutive late layers."""
    Hs = np.asarray(Hs, dtype=np.float64)
    K = Hs.shape[0] - 1
    total = np.zeros(Hs.shape[1], dtype=np.float64)
    for l in range(1, K + 1):
        diff = Hs[l] - Hs[l - 1]
        total += np.sqrt(np.sum(diff * diff, axis=1))
    return total / K


# --------------------------------------------------------------------------
# step 4: normalise and fuse
# --------------------------------------------------------------------------
def minmax(s: np.ndarray) -> np.ndarray:
    lo, hi = s.min(), s.max()
    if hi == lo:
        return np.zeros_like(s)
    return (s - lo) / (hi - lo)


def fuse(s_query: np.ndarray, s_act: Optional[np.ndarray], lam: float) -> np.ndarray:
    """Fused score; with no activity term the fused score is the normalised query score."""
    if s_act is None:
        return minmax(s_query)
    return lam * minmax(s_query) + (1.0 - lam) * minmax(s_act)


# --------------------------------------------------------------------------
# steps 5 / 7: ranking decisions
# --------------------------------------------------------------------------
def decision_values(s: np.ndarray) -> np.ndarray:
    """Scores as the decision sees them: rounded to float32."""
    return np.asarray(s, dtype=np.float64).astype(np.float32)


def top_indices(s: np.ndarray, m: int) -> np.ndarray:
    """Indices of the m largest entries (ties -> lower index), returned ascending."""
    v = decision_values(s)
    order = np.argsort(-v.astype(np.float64), kind="stable")  # stable => lower index first on ties
    return np.sort(order[:m]).astype(np.int32)


def cut_margin(s: np.ndarray, m: int) -> float:
    """Relative gap between the last kept and the first dropped value (inf if nothing dropped)."""
    v = np.sort(decision_values(s).astype(np.float64))[::-1]
    if m >= v.size:
        return float("inf")
    scale = max(abs(v[0]), abs(v[-1]), 1e-300)
    return float((v[m - 1] - v[m]) / scale)


# --------------------------------------------------------------------------
# step 6: low-rank subspace energy
# --------------------------------------------------------------------------
def subspace_energy(Zrows: np.ndarray, r: int):
    """Zrows is [M, d] (row i = z_i, i.e. Z_M transposed).  Returns (c, sigma).

    Z_M = U S V^T with Z_M = Zrows^T (d x M); c_i = sum_{k<r} (S_k V_ik)^2.
    """
    Zm = np.asarray(Zrows, dtype=np.float64).T           # d x M
    U, S, Vt = np.linalg.svd(Zm, full_matrices=False)     # S descending
    VS = Vt[:r, :].T * S[:r][None, :]                     # (V_r Sigma_r), M x r
    return np.sum(VS * VS, axis=1), S


def greedy_residual(Zrows: np.ndarray, k: int):
    """Variant selector: k greedy picks, each the token with the largest residual.

    Pivoted Cholesky of G = Z Z^T:  rho_i <- G_ii; repeat: p = argmax rho (on the
    float32-rounded values, ties -> lower index), l = (G[:,p] - L L[p,:]^T)/sqrt(rho_p),
    rho <- rho - l^2.  Returns (pick_order, resid) where resid[t] is rho_p at pick t.
    """
    Z = np.asarray(Zrows, dtype=np.float64)
    M = Z.shape[0]
    G = Z @ Z.T
    rho = np.diag(G).copy()
    L = np.zeros((M, k), dtype=np.float64)
    picked = np.zeros(M, dtype=bool)
    order = np.empty(k, dtype=np.int32)
    resid = np.empty(k, dtype=np.float64)
    for t in range(k):
        cand = np.where(picked, -np.inf, rho)
        p = int(np.argmax(decision_values(cand)))          # first maximum = lowest index
        order[t], resid[t] = p, rho[p]
        picked[p] = True
        piv = max(rho[p], 0.0)
        if piv > 0.0:
            col = (G[:, p] - L[:, :t] @ L[p, :t]) / np.sqrt(piv)
        else:
            col = np.zeros(M)
        L[:, t] = col
        rho = rho - col * col
    return order, resid


# --------------------------------------------------------------------------
# whole path
# --------------------------------------------------------------------------
def score(X, hidden, Q, Wq, Wk, p: Params) -> Dict[str, np.ndarray]:
    """Steps 1-4 for one image.  X [N,d], hidden [K+1,N,d] or None, Q [T,d]."""
    Ev, Eq = embed(X, Wk), embed(Q, Wq)
    if p.rel_mode == REL_COSINE_MAX:
        s_query = query_score_cosine(Ev, Eq)
    else:
        s_query = query_score_attention(Ev, Eq, p.n_heads)
    s_act = None if hidden is None or np.shape(hidden)[0] < 2 else activity_score(hidden)
    s_fused = fuse(s_query, s_act, p.lam)
    return {"s_query": s_query, "s_act": s_act, "s_fused": s_fused}


_MASK64 = (1 << 64) - 1


def mix64(x: int) -> int:
    """The output function of the SplitMix64 generator (Steele, Lea, Flood 2014) on a 64-bit word."""
    z = x & _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def random_scores(seed: int, image: int, n_tokens: int) -> np.ndarray:
    """Counter-based uniform scores in [0, 1) with 24 bits, one per (seed, image, token).

    word = seed * 0x9E3779B97F4A7C15 + (image << 32 | token) + 0x632BE59BD9B4E019 (mod 2^64); the score is
    the top 24 bits of mix64(word) times 2^-24, which float32 holds exactly.  Keeping the k largest (ties ->
    lower index) draws k tokens uniformly without replacement.
    """
    out = np.empty(n_tokens, dtype=np.float64)
    for i in range(n_tokens):
        word = (seed * 0x9E3779B97F4A7C15 + ((image << 32) | i) + 0x632BE59BD9B4E019) & _MASK64
        out[i] = (mix64(word) >> 40) * 2.0 ** -24
    return out


def select(X, s_fused, p: Params, image: int = 0) -> Dict[str, np.ndarray]:
    """Steps 5-7 for one image, from a fused score vector (`image`: its index in the batch, used by LR_RANDOM)."""
    X = np.asarray(X, dtype=np.float64)
    k, M, r = p.resolved(X.shape[0])
    if p.lr_mode == LR_RANDOM:
        u = random_scores(p.seed, image, X.shape[0])
        return {"idx": top_indices(u, k).astype(np.int32), "random_scores": u}
    if p.lr_mode == LR_SCORE_TOPK:
        return {"idx": top_indices(s_fused, k).astype(np.int32), "idx_m": top_indices(s_fused, M),
                "margin_topk": cut_margin(s_fused, k)}
    idx_m = top_indices(s_fused, M)
    Z = X[idx_m]
    out = {"idx_m": idx_m, "margin_topm": cut_margin(s_fused, M)}
    if p.lr_mode == LR_ENERGY_TOPK:
        c, sigma = subspace_energy(Z, r)
        keep_local = top_indices(c, k)
        out.update(c=c, sigma=sigma, margin_topk=cut_margin(c, k),
                   sigma_gap=float((sigma[r - 1] ** 2 - sigma[r] ** 2) / sigma[r - 1] ** 2) if r < sigma.size else float("inf"))
    else:
        order, resid = greedy_residual(Z, k)
        keep_local = np.sort(order).astype(np.int32)
        out.update(pick_order=idx_m[order], resid=resid)
    out["idx"] = idx_m[keep_local].astype(np.int32)
    return out


def reduce(X, hidden, Q, Wq, Wk, p: Params, image: int = 0) -> Dict[str, np.ndarray]:
    """Steps 1-8 for one image; 'tokens' are rows of X (the stored features, not embeddings)."""
    sc = score(X, hidden, Q, Wq, Wk, p)
    # the fused score crosses the library boundary as float32; selection sees those bits
    se = select(X, decision_values(sc["s_fused"]), p, image)
    out = dict(sc)
    out.update(se)
    out["tokens"] = np.asarray(X)[se["idx"]]
    return out
