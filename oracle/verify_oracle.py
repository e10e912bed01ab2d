"""CPU oracle for the speculative verification arithmetic over the vocabulary.

TEST INFRASTRUCTURE ONLY (imported by tests and by the benchmark's CPU baseline; the product path never
calls it and shares no code with it).  Plain float64 NumPy, written from the paper's Section II-A
("Collaborative VLM Inference Pipeline"): the softmax distributions of the draft and the target logits, the
acceptance probability of a drafted token, and the residual distribution a correction is drawn from after
the first rejection.

Per sequence with L drafted positions tau = 0..L-1 over a vocabulary of V words:

    p_d(w|tau) = softmax(z_d[tau])_w,  p_t(w|tau) = softmax(z_t[tau])_w          (the two softmax equations)
    alpha_tau  = min(1, p_t(y_tau|tau) / p_d(y_tau|tau))                          (acceptance equation)
    position tau is accepted iff u_tau < alpha_tau, u_tau uniform in [0, 1)
    n_acc = number of accepted positions before the first rejection
    if n_acc < L: the correction is drawn from
    r(w) = max(p_t(w) - p_d(w), 0) / sum_u max(p_t(u) - p_d(u), 0)  at tau = n_acc (residual equation)

Readings where the paper is silent: the uniforms are inputs (the paper names no generator); the accept test
compares the float32 uniform with alpha rounded to float32, the precision in which the library returns
alpha; the draw from r is by inverse CDF in vocabulary order: the smallest w whose cumulative residual mass
exceeds u_res times the total; a residual with zero mass (p_t == p_d, where a rejection has probability
zero) yields argmax p_t; when every position is accepted no correction exists (-1): the bonus token the
paper mentions needs the target logits of one more position, which this step does not have.

Parity status: pinned by tests/test_verify_oracle_pins.py (scipy softmax, closed forms, the identity that
accept-or-resample reproduces p_t exactly, brute-force inverse CDF).
"""
from __future__ import annotations

from typing import Dict

import numpy as np


def softmax(z: np.ndarray) -> np.ndarray:
    """softmax over the last axis (the two softmax equations of Sec. II-A), shifted by the row maximum."""
    z = np.asarray(z, dtype=np.float64)
    e = np.exp(z - z.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def accept_prob(pt: np.ndarray, pd: np.ndarray, tok: int) -> float:
    """alpha = min(1, p_t(y) / p_d(y)) (acceptance equation); a token the draft gives zero mass is accepted."""
    if pd[tok] <= 0.0:
        return 1.0
    return float(min(1.0, pt[tok] / pd[tok]))


def residual_weights(pt: np.ndarray, pd: np.ndarray) -> np.ndarray:
    """Unnormalised residual max(p_t - p_d, 0) (numerator of the residual equation)."""
    return np.maximum(pt - pd, 0.0)


def inverse_cdf(weights: np.ndarray, u: float) -> int:
    """Smallest index w with sum(weights[:w+1]) > u * sum(weights); weights >= 0 with positive total."""
    c = np.cumsum(weights)            # sequential, index order
    target = float(u) * c[-1]
    w = int(np.searchsorted(c, target, side="right"))
    return min(w, len(weights) - 1)


def verify(zt: np.ndarray, zd: np.ndarray, tok: np.ndarray, u_acc: np.ndarray, u_res: float) -> Dict[str, object]:
    """One sequence: zt, zd [L, V] logits, tok [L] drafted tokens, u_acc [L] and u_res uniforms in [0, 1)."""
    zt = np.asarray(zt, dtype=np.float64)
    zd = np.asarray(zd, dtype=np.float64)
    L = zt.shape[0]
    pt, pd = softmax(zt), softmax(zd)
    alpha = np.array([accept_prob(pt[t], pd[t], int(tok[t])) for t in range(L)])
    accepted = np.asarray(u_acc, dtype=np.float32) < alpha.astype(np.float32)
    n_acc = L if accepted.all() else int(np.argmin(accepted))
    out: Dict[str, object] = {"alpha": alpha, "n_acc": n_acc, "corr": -1}
    if n_acc < L:
        w = residual_weights(pt[n_acc], pd[n_acc])
        out["residual_mass"] = float(w.sum())
        out["corr"] = inverse_cdf(w, u_res) if w.sum() > 0.0 else int(np.argmax(pt[n_acc]))
        out["weights"] = w
    return out
