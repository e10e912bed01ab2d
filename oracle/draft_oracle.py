"""CPU oracle for the draft-side vocabulary pass: margin gate and bonus-token candidates.

TEST INFRASTRUCTURE ONLY (imported by tests and by the benchmark's CPU baseline; the product path never
calls it and shares no code with it).  Plain float64 NumPy, written from the paper's Section III-B
("Margin-Based Gating": the margin and the gating equations) and Section III-C ("Parallel Branching": the
fan-out equation and the candidate rule).

Per drafted position tau with draft logits z_d [V] and drafted token y:

    p_d = softmax(z_d)
    m   = p_(1) - p_(2), the two largest probabilities                         (margin equation)
    g   = 0 if m >= gamma else 1                                                (gating equation)
    F_j = ceil(F_0 * rho^j), j the position inside the drafted segment          (fan-out equation)
    candidates = the F_j words with the largest draft logits, the drafted token left out

Readings where the paper is silent: the gate compares the margin rounded to float32 with gamma as float32
(the precision the library returns the margin in); equal logits are ordered by the lower word index, in the
top-2 and in the candidate list; candidates are listed by descending logit; F_j is the exact ceiling of F_0 rho^j for the decimal
rho (rational arithmetic) and a vocabulary with fewer than F_j other words yields fewer candidates.

Parity status: pinned by tests/test_draft_oracle_pins.py (closed forms for two words and for one boosted
word, the fan-out sequence for rho = 1/2, brute-force repeated argmax, invariants).
"""
from __future__ import annotations

import math
from fractions import Fraction
from typing import Dict, List

import numpy as np


def softmax(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=np.float64)
    e = np.exp(z - z.max())
    return e / e.sum()


def margin(zd: np.ndarray) -> float:
    """m = p_(1) - p_(2) of softmax(zd) (margin equation, Sec. III-B)."""
    p = np.sort(softmax(zd))
    return float(p[-1] - p[-2])


def gate(m: float, gamma: float) -> int:
    """g = 0 (commit locally) if m >= gamma, else 1 (verify) (gating equation), compared in float32."""
    return 0 if np.float32(m) >= np.float32(gamma) else 1


def fanout(f0: int, rho: float, n: int) -> List[int]:
    """F_j = ceil(F_0 rho^j), j = 0..n-1 (fan-out equation, Sec. III-C), in exact rational arithmetic: rho is
    taken as the decimal number its shortest representation spells (0.1 is one tenth), so an exact integer is never
    tipped over by the binary rounding of rho or of the power."""
    q = Fraction(repr(float(rho)))
    return [int(math.ceil(f0 * q ** j)) for j in range(n)]


def candidates(zd: np.ndarray, y: int, f: int) -> np.ndarray:
    """The f words with the largest draft logits other than y, by descending logit, lower index first on ties."""
    zd = np.asarray(zd, dtype=np.float64)
    order = np.argsort(-zd, kind="stable")
    order = order[order != y]
    return order[:f].astype(np.int64)


def draft_pass(zd: np.ndarray, tok: np.ndarray, f0: int, rho: float, gamma: float) -> Dict[str, object]:
    """One sequence: zd [L, V] draft logits, tok [L] drafted tokens."""
    zd = np.asarray(zd, dtype=np.float64)
    L = zd.shape[0]
    F = fanout(f0, rho, L)
    m = np.array([margin(zd[t]) for t in range(L)])
    return {"margin": m, "gate": np.array([gate(x, gamma) for x in m], dtype=np.int32), "fanout": F,
            "cand": [candidates(zd[t], int(tok[t]), F[t]) for t in range(L)]}
