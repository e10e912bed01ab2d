"""GPU parity at the full sizes of the five benchmark workloads, in the launch configuration
the benchmark times (whole batch in one call).  Images are independent, so the oracle checks
every image of every workload (workload 5: all 64 images, in both pipelines).

Bars as in test_gpu_parity.py: kept indices bit-exact, scores within 1e-5 (fp32) / 2e-2 (bf16).
"""
import gc
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import covspec_inputs as I
from oracle import covspec_oracle as O
from tests import util as U

pytestmark = pytest.mark.gpu

SAMPLE = {1: [0], 2: [0], 3: list(range(8)), 4: list(range(4)), 5: list(range(64))}
_cache = {}


@pytest.fixture(scope="module")
def C():
    import paper_2605_02218_amd as C
    C.load_library()
    return C


def _workload(cid):
    """Generate (and keep for the two pipelines of) one workload at a time."""
    if cid not in _cache:
        _cache.clear()
        gc.collect()
        import torch
        torch.cuda.empty_cache()
        w = I.WORKLOADS[cid]
        batch = U.gen_batch(w, workers=16)
        _cache[cid] = (w, batch, U.upload(batch, w.dtype))
    return _cache[cid]


def _progress(it, what):
    """Pass the items through, with a line every eight so that a long oracle run shows it is alive."""
    for n, item in enumerate(it, 1):
        if n % 8 == 0:
            print("%s: %d images done" % (what, n), flush=True)
        yield item


def _cpu(t):
    return t.detach().cpu().numpy()


@pytest.mark.parametrize("modes", [(0, 0), (1, 1)], ids=["paper", "variant"])
@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_full_size_reduce_matches_oracle(C, cid, modes):
    import torch
    w, batch, dev = _workload(cid)
    p = U.lib_params(C, w, w.batch, rel_mode=modes[0], lr_mode=modes[1])
    ws = C.alloc_workspace(p)
    idx, tok = C.reduce(p, dev["X"], dev["hidden"], dev["Q"], dev["Wq"], dev["Wk"], workspace=ws)
    sq, sa, sf = C.score(p, dev["X"], dev["hidden"], dev["Q"], dev["Wq"], dev["Wk"], workspace=ws)
    sel = C.select(p, dev["X"], sf, workspace=ws)
    torch.cuda.synchronize()
    idx_h, sq, sa, sf = _cpu(idx), _cpu(sq), _cpu(sa), _cpu(sf)
    np.testing.assert_array_equal(_cpu(sel["idx"]), idx_h)          # the three entry points agree

    # properties that hold for every image at any size
    assert idx_h.shape == (w.batch, w.keep_k) and idx_h.min() >= 0 and idx_h.max() < w.n_tokens
    assert np.all(np.diff(idx_h, axis=1) > 0)
    tok_bits = tok.view(torch.int16 if w.dtype == I.BF16 else torch.float32)
    X_bits = dev["X"].view(torch.int16 if w.dtype == I.BF16 else torch.float32)
    gathered = torch.gather(X_bits, 1, idx.long()[:, :, None].expand(-1, -1, w.d_model))
    assert bool((tok_bits == gathered).all())
    idx_m_h = _cpu(sel["idx_m"])
    assert all(np.isin(idx_h[b], idx_m_h[b]).all() for b in range(w.batch))
    if modes[0] == 1:
        np.testing.assert_allclose(sq.astype(np.float64).sum(axis=1), 1.0, atol=1e-4)

    worst = {}
    assert SAMPLE[cid] == list(range(w.batch))          # every image of the batch meets the oracle
    op = U.oracle_params(w, rel_mode=modes[0], lr_mode=modes[1])
    with ThreadPoolExecutor(max_workers=4) as ex:      # the oracle's BLAS calls release the interpreter lock
        refs = ex.map(lambda b: U.oracle_image(w, batch, b, op), SAMPLE[cid])
        refs = [r for r in _progress(refs, "c%d %s oracle" % (cid, modes))]
    for b, ref in zip(SAMPLE[cid], refs):
        tag = "c%d img %d" % (cid, b)
        worst["s_query"] = max(worst.get("s_query", 0), U.assert_scores_close(sq[b], ref["s_query"], w.dtype, tag + " s_query"))
        worst["s_act"] = max(worst.get("s_act", 0), U.assert_scores_close(sa[b], ref["s_act"], w.dtype, tag + " s_act"))
        worst["s_fused"] = max(worst.get("s_fused", 0), U.assert_scores_close(sf[b], ref["s_fused"], w.dtype, tag + " s_fused"))
        np.testing.assert_array_equal(_cpu(sel["idx_m"])[b], ref["idx_m"],
                                      err_msg="%s idx_m, margin %r" % (tag, ref["margin_topm"]))
        if modes[1] == 0:
            worst["c"] = max(worst.get("c", 0), U.assert_scores_close(_cpu(sel["c"])[b], ref["c"], w.dtype, tag + " c"))
        else:
            np.testing.assert_array_equal(_cpu(sel["pick_order"])[b], ref["pick_order"], err_msg=tag + " pick order")
            worst["resid"] = max(worst.get("resid", 0), U.assert_scores_close(_cpu(sel["resid"])[b], ref["resid"], w.dtype, tag + " resid"))
        np.testing.assert_array_equal(idx_h[b], ref["idx"], err_msg="%s idx, margins topm=%r topk=%r gap=%r" % (
            tag, ref["margin_topm"], ref.get("margin_topk"), ref.get("sigma_gap")))
    print("c%d %s worst rel err: %s" % (cid, modes, {k: "%.2e" % v for k, v in worst.items()}), flush=True)
