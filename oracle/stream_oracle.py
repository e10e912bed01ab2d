"""CPU oracle for the streaming form of the visual token selection.

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's CPU baseline, never by
the product path, with which it shares no code.  float64 NumPy.

The paper (Sec. III-A) selects the tokens of one image at once.  For video whose frames arrive one by
one this module states the frame-by-frame form that the library's streaming entry point implements; it
is NOT in the paper, and is defined so that every frame is exactly one application of the paper's
low-rank step (Sec. III-A.3: stacking, rank-r SVD, energy, keep the largest) to a candidate set:

  state after a frame: at most k kept tokens (feature rows and caller-side ids), in candidate order;
  a frame arrives with N_f tokens and their fused scores (Sec. III-A fusion equation, normalised over
  the frame by whoever computed them):
    1. the M_f tokens of the frame with the largest score are pre-selected (ascending position);
    2. candidates = kept tokens, then the pre-selected ones (n_C = n_keep + M_f rows);
    3. n_C <= k: all candidates are kept.  Otherwise c_i = energy of candidate i in the top-r singular
       subspace of the candidate matrix, and the k candidates with the largest c (decided on float32
       values, ties to the earlier candidate) are kept, in candidate order.

Nothing is carried but the rows themselves, so the Gram matrix of the candidates is recomputed from
scratch at every frame (inside the SVD).  The library instead carries the kept tokens' Gram matrix and
computes only the rows of the arriving tokens; the parity tests therefore also check that shortcut.

Every step is a function of covspec_oracle that tests/test_oracle_pins.py pins; what is new here is
their composition, pinned by tests/test_stream_oracle_pins.py.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List

import numpy as np

from . import covspec_oracle as O


@dataclass
class StreamState:
    rows: np.ndarray                      # [n_keep, d] float64
    ids: np.ndarray                       # [n_keep] int64, caller-side token ids
    history: List[Dict[str, np.ndarray]] = field(default_factory=list)


def empty_state(d_model: int) -> StreamState:
    return StreamState(np.zeros((0, d_model)), np.zeros((0,), dtype=np.int64))


def stream_step(state: StreamState, X_frame: np.ndarray, s_fused: np.ndarray, id_base: int, frame_m: int,
                keep_k: int, rank_r: int) -> Dict[str, np.ndarray]:
    """One arriving frame; updates `state` and returns what was decided.

    X_frame [N_f, d], s_fused [N_f].  Returned: idx_f (pre-selected positions), c (energies of the n_C
    candidates, None when all are kept), sel (kept candidate positions, ascending), ids (kept ids),
    margin_topm / margin_topk (relative gaps at the two cuts, for choosing test inputs that have no
    near-tie).
    """
    X = np.asarray(X_frame, dtype=np.float64)
    idx_f = O.top_indices(s_fused, frame_m)
    cand_rows = np.concatenate([state.rows, X[idx_f]], axis=0)
    cand_ids = np.concatenate([state.ids, id_base + idx_f.astype(np.int64)])
    n_c = cand_rows.shape[0]
    out = {"idx_f": idx_f, "margin_topm": O.cut_margin(s_fused, frame_m), "c": None, "margin_topk": float("inf")}
    if n_c <= keep_k:
        sel = np.arange(n_c, dtype=np.int32)
    else:
        c, sigma = O.subspace_energy(cand_rows, rank_r)
        sel = O.top_indices(c, keep_k)
        out["c"] = c
        out["margin_topk"] = O.cut_margin(c, keep_k)
        out["sigma_gap"] = float((sigma[rank_r - 1] - sigma[rank_r]) / sigma[0]) if rank_r < sigma.size else float("inf")
    state.rows = cand_rows[sel]
    state.ids = cand_ids[sel]
    out["sel"] = sel
    out["ids"] = state.ids.copy()
    state.history.append(out)
    return out
