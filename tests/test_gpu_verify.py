"""GPU parity of covspec_verify (paper Sec. II-A: acceptance probability, first rejection, residual draw)
against oracle/verify_oracle.py, element by element on the same seeded logits.

alpha is compared within 1e-5 relative (fp32 exponentials in the streaming pass, fp64 combination);
n_accept and the correction are integers and compared exactly.  Both are decided by a floating-point
comparison, so each case first checks ON THE ORACLE'S VALUES that no decision sits inside the rounding band
(|u - alpha| > 1e-5 alpha; the residual's cumulative sum clears u * total by more than 1e-9 of the total on
both sides of the drawn word): inside that band either answer would be a correct rounding.
"""
import numpy as np
import pytest

import covspec_inputs as I
from oracle import verify_oracle as VO

pytestmark = pytest.mark.gpu

ALPHA_RTOL = 1e-5


def _dev(a, dtype=None):
    import torch
    if dtype == I.BF16:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)
    if dtype == I.FP16:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.float16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _run(d, dtype, want_alpha=True):
    import torch
    import paper_2605_02218_amd as C
    S, L, V = d["zt"].shape
    p = C.VerifyParams(n_seq=S, n_draft=L, vocab=V, dtype=dtype)
    n_acc, corr, alpha = C.verify(p, _dev(d["zt"], dtype), _dev(d["zd"], dtype), _dev(d["tok"]), _dev(d["u_acc"]),
                                  _dev(d["u_res"]), want_alpha=want_alpha)
    torch.cuda.synchronize()
    return n_acc.cpu().numpy(), corr.cpu().numpy(), None if alpha is None else alpha.cpu().numpy()


def _check(d, dtype, n_acc, corr, alpha, seqs=None):
    S, L, V = d["zt"].shape
    for s in (range(S) if seqs is None else seqs):
        zt, zd = I.as_f64(d["zt"][s], dtype), I.as_f64(d["zd"][s], dtype)
        o = VO.verify(zt, zd, d["tok"][s], d["u_acc"][s], d["u_res"][s])
        a = o["alpha"]
        # decisions outside the rounding band (a property of the seeded inputs, checked on the oracle)
        assert np.all(np.abs(d["u_acc"][s].astype(np.float64) - a)[: min(o["n_acc"] + 1, L)] > ALPHA_RTOL * a[: min(o["n_acc"] + 1, L)]), s
        if alpha is not None:
            np.testing.assert_allclose(alpha[s], a, rtol=ALPHA_RTOL, atol=0, err_msg="alpha, sequence %d" % s)
        assert n_acc[s] == o["n_acc"], (s, n_acc[s], o["n_acc"])
        if o["n_acc"] < L and o.get("residual_mass", 0.0) > 0.0:
            c = np.cumsum(o["weights"])
            target = float(d["u_res"][s]) * c[-1]
            w = o["corr"]
            lower = c[w - 1] if w > 0 else 0.0
            band = 1e-9 * c[-1]
            assert c[w] - target > band and (target - lower > band or target == 0.0), s
        assert corr[s] == o["corr"], (s, corr[s], o["corr"])


@pytest.mark.parametrize("dtype,V", [(I.BF16, 4392), (I.FP32, 4100), (I.BF16, 8), (I.FP32, 4), (I.BF16, 2048 * 3), (I.FP16, 4392),
                                     (I.FP16, 8)])
def test_verify_matches_oracle_small(dtype, V):
    """Several chunks with a ragged last one (4392 = 2 * 2048 + 296), exact multiples, and the smallest widths."""
    d = I.make_verify_batch(6, 4, V, dtype, seed=V, copy_rows=1)
    n_acc, corr, alpha = _run(d, dtype)
    assert n_acc[0] == 4 and corr[0] == -1 and np.all(alpha[0] == 1.0)    # draft == target: always accepted
    _check(d, dtype, n_acc, corr, alpha)


@pytest.mark.parametrize("S,L", [(1, 1), (1, 8), (37, 3), (300, 1)])
def test_verify_batch_shapes(S, L):
    """One row (64 chunks of the row), many sequences (one chunk per row), odd counts."""
    d = I.make_verify_batch(S, L, 8200, I.BF16, seed=100 * S + L, disagreement=0.9)
    n_acc, corr, alpha = _run(d, I.BF16)
    _check(d, I.BF16, n_acc, corr, alpha)
    n2, c2, none = _run(d, I.BF16, want_alpha=False)      # alpha_out is optional
    assert none is None and np.array_equal(n2, n_acc) and np.array_equal(c2, corr)


def test_verify_edge_uniforms_and_tokens():
    """u_res at 0 and just below 1 (first / last word with residual mass), drafted tokens at both ends of the
    vocabulary, and a first-position rejection."""
    dtype, V = I.FP32, 5000
    d = I.make_verify_batch(8, 4, V, dtype, seed=77, disagreement=1.2)
    d["tok"][0, :] = 0
    d["tok"][1, :] = V - 1
    d["u_acc"][2, 0] = np.float32(0.99999994)          # rejected at once unless alpha == 1
    d["u_acc"][3, :] = 0.0                              # every position accepted (alpha > 0)
    d["u_res"][2] = 0.0
    d["u_res"][4] = np.float32(0.99999994)
    d["u_acc"][4, 1] = np.float32(0.99999994)
    d["u_res"][5] = 0.0
    d["u_acc"][5, 2] = np.float32(0.99999994)
    n_acc, corr, alpha = _run(d, dtype)
    assert n_acc[3] == 4 and corr[3] == -1
    for s in (2, 4, 5):
        zt, zd = I.as_f64(d["zt"][s], dtype), I.as_f64(d["zd"][s], dtype)
        o = VO.verify(zt, zd, d["tok"][s], d["u_acc"][s], d["u_res"][s])
        assert n_acc[s] == o["n_acc"] and corr[s] == o["corr"], s
        nz = np.nonzero(o["weights"])[0]
        if d["u_res"][s] == 0.0:
            assert corr[s] == nz[0]
    _check(d, dtype, n_acc, corr, alpha, seqs=(0, 1, 3, 6, 7))


def test_verify_masked_words_and_large_logits():
    """A padded vocabulary (-inf logits on the tail and on a whole leading chunk) and logits far from zero:
    the shifted exponentials must neither overflow nor produce NaN."""
    dtype, V = I.BF16, 6144
    d = I.make_verify_batch(5, 3, V, dtype, seed=5, disagreement=0.8)
    zt, zd = I.as_f32(d["zt"], dtype), I.as_f32(d["zd"], dtype)
    zt[:, :, V - 300:] = -np.inf
    zd[:, :, V - 300:] = -np.inf
    zt[1, :, :2048] = -np.inf                         # a whole chunk masked
    zd[1, :, :2048] = -np.inf
    zt[2] = zt[2] * 20.0 + 300.0                      # large offset and spread
    zd[2] = zd[2] * 20.0 - 250.0
    d["zt"], d["zd"] = I.store(zt, dtype), I.store(zd, dtype)
    g = np.random.default_rng(9).gumbel(size=zd.shape)
    d["tok"] = np.argmax(I.as_f64(d["zd"], dtype) + g, axis=2).astype(np.int32)   # drafted words are unmasked
    n_acc, corr, alpha = _run(d, dtype)
    assert np.all(np.isfinite(alpha))
    assert np.all((corr < V - 300) & ((corr >= 0) | (n_acc == 3)))
    _check(d, dtype, n_acc, corr, alpha)


def test_verify_rejection_with_empty_residual_takes_the_argmax():
    """u = 1 lies outside the contract [0, 1) but forces a rejection where p_t == p_d: the residual has no mass
    and the correction is the target's most likely word (lowest index on ties)."""
    dtype, V = I.BF16, 4104
    d = I.make_verify_batch(3, 2, V, dtype, seed=11, copy_rows=3)
    d["u_acc"][:, 0] = 1.0
    n_acc, corr, alpha = _run(d, dtype)
    assert np.all(n_acc == 0) and np.all(alpha == 1.0)
    for s in range(3):
        z = I.as_f64(d["zt"][s, 0], dtype)
        assert corr[s] == int(np.argmax(z))
        o = VO.verify(I.as_f64(d["zt"][s], dtype), I.as_f64(d["zd"][s], dtype), d["tok"][s], d["u_acc"][s], d["u_res"][s])
        assert o["corr"] == corr[s] and o["n_acc"] == 0


def test_verify_full_vocabulary_batch():
    """The benchmark's shape: 64 sequences of 8 drafted positions over 151,936 words, bf16, every sequence
    against the oracle."""
    dtype = I.BF16
    S, L, V = 64, 8, I.VERIFY_VOCAB
    d = I.make_verify_batch(S, L, V, dtype, seed=2024, copy_rows=2)
    n_acc, corr, alpha = _run(d, dtype)
    assert 0 < (n_acc == L).sum() < S                   # the workload has both outcomes
    _check(d, dtype, n_acc, corr, alpha)
