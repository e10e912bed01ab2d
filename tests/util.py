"""Shared helpers for the parity tests: input upload, oracle driving, tolerances."""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import Dict, Iterable, Optional

import numpy as np

import covspec_inputs as I
from oracle import covspec_oracle as O

# score tolerance: relative, with the denominator floored at 1e-3 of the largest reference magnitude
TOL = {I.FP32: 1e-5, I.BF16: 2e-2}


def gen_batch(w: I.Workload, images: Optional[Iterable[int]] = None, workers: int = 8) -> Dict[str, np.ndarray]:
    images = list(range(w.batch)) if images is None else list(images)
    with ThreadPoolExecutor(max_workers=min(workers, len(images))) as ex:
        per = list(ex.map(lambda b: I.make_image(w, b), images))
    out = {k: np.stack([p[k] for p in per]) for k in ("X", "Q", "hidden")}
    out.update(I.make_weights(w))
    return out


def to_device(a: np.ndarray, dtype: int):
    import torch
    if dtype == I.BF16:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def upload(batch: Dict[str, np.ndarray], dtype: int):
    return {k: to_device(v, dtype) for k, v in batch.items()}


def oracle_params(w: I.Workload, rel_mode=0, lr_mode=0, **over) -> O.Params:
    kw = dict(n_heads=w.n_heads, rel_mode=rel_mode, lr_mode=lr_mode, preselect_m=w.preselect_m,
              rank_r=w.rank_r, keep_k=w.keep_k, lam=w.lam)
    kw.update(over)
    return O.Params(**kw)


def lib_params(C, w: I.Workload, batch: int, rel_mode=0, lr_mode=0, **over):
    kw = dict(batch=batch, n_tokens=w.n_tokens, d_model=w.d_model, n_query=w.n_query, n_heads=w.n_heads,
              n_act_layers=w.n_act_layers, dtype=w.dtype, rel_mode=rel_mode, lr_mode=lr_mode,
              preselect_m=w.preselect_m, rank_r=w.rank_r, keep_k=w.keep_k, lam=w.lam)
    kw.update(over)
    return C.Params(**kw)


def oracle_image(w: I.Workload, batch: Dict[str, np.ndarray], b: int, p: O.Params, use_hidden=True,
                 use_wq=True, use_wk=True):
    """Run the oracle on image b of a generated batch (inputs exactly as stored)."""
    X = I.as_f64(batch["X"][b], w.dtype)
    Q = I.as_f64(batch["Q"][b], w.dtype)
    H = I.as_f64(batch["hidden"][b], w.dtype) if use_hidden else None
    Wq = I.as_f64(batch["Wq"], w.dtype) if use_wq else None
    Wk = I.as_f64(batch["Wk"], w.dtype) if use_wk else None
    return O.reduce(X, H, Q, Wq, Wk, p, image=b)


def assert_scores_close(got: np.ndarray, ref: np.ndarray, dtype: int, what: str, tol: Optional[float] = None):
    tol = TOL[dtype] if tol is None else tol
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    denom = np.maximum(np.abs(ref), np.abs(ref).max() * 1e-3)
    err = np.abs(got - ref) / np.maximum(denom, 1e-300)
    worst = int(np.argmax(err))
    assert err.max() <= tol, "%s: rel err %.3e at %d (got %r ref %r), tol %.1e" % (
        what, err.max(), worst, got.flat[worst], ref.flat[worst], tol)
    return float(err.max())
