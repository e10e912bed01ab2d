"""GPU parity of covspec_draft_gate (paper Sec. III-B margin gate, Sec. III-C bonus-token candidates) against
oracle/draft_oracle.py on the same seeded logits.

Candidates are word indices: compared exactly, in order (descending logit, lower word first among equals).
The margin is compared within 1e-5 relative plus 2e-6 absolute (fp32 exponentials in the streaming sum bound
each probability to ~1e-6 relative; probabilities are at most 1).  The gate is decided by a floating-point
comparison, so each case first checks on the ORACLE's margin that it is not within that error of gamma.
"""
import numpy as np
import pytest

import covspec_inputs as I
from oracle import draft_oracle as DO

pytestmark = pytest.mark.gpu


def _dev(a, dtype=None):
    import torch
    if dtype == I.BF16:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)
    if dtype == I.FP16:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.float16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _run(zd, tok, dtype, f0, rho, gamma):
    import torch
    import paper_2605_02218_amd as C
    S, L, V = zd.shape
    p = C.DraftParams(n_seq=S, n_draft=L, vocab=V, dtype=dtype, fanout0=f0, rho=rho, gamma=gamma)
    margin, gate, cand = C.draft_gate(p, _dev(zd, dtype), _dev(tok))
    torch.cuda.synchronize()
    return margin.cpu().numpy(), gate.cpu().numpy(), None if cand is None else cand.cpu().numpy()


def _check(zd, tok, dtype, f0, rho, gamma, margin, gate, cand, seqs=None):
    S, L, V = zd.shape
    rho32, gamma32 = float(rho), float(np.float32(gamma))      # rho is a double in the parameter block
    for s in (range(S) if seqs is None else seqs):
        o = DO.draft_pass(I.as_f64(zd[s], dtype), tok[s], f0, rho32, gamma32)
        tol = 1e-5 * o["margin"] + 2e-6
        assert np.all(np.abs(o["margin"] - gamma32) > tol), "a margin of the seeded inputs sits on the threshold"
        assert np.all(np.abs(margin[s] - o["margin"]) <= tol), (s, margin[s], o["margin"])
        assert np.array_equal(gate[s], o["gate"]), s
        for t in range(L):
            want = np.full(f0, -1, dtype=np.int64)
            want[:len(o["cand"][t])] = o["cand"][t]
            assert np.array_equal(cand[s, t], want), (s, t, cand[s, t], want)


@pytest.mark.parametrize("dtype,V", [(I.BF16, 2 * 8192 + 520), (I.FP32, 8192 + 36), (I.BF16, 8192), (I.BF16, 8), (I.FP32, 4), (I.BF16, 264),
                                     (I.FP16, 2 * 8192 + 520), (I.FP16, 16)])
def test_draft_gate_matches_oracle_small(dtype, V):
    """Several chunks with a ragged last one, an exact chunk, and vocabularies smaller than the candidate count
    (fewer quads with data than K: the block-wide fallback)."""
    d = I.make_verify_batch(3, 5, V, dtype, seed=V + 1)
    m, g, c = _run(d["zd"], d["tok"], dtype, 6, 0.6, 0.3)
    _check(d["zd"], d["tok"], dtype, 6, 0.6, 0.3, m, g, c)


@pytest.mark.parametrize("f0,rho", [(1, 0.5), (32, 0.9), (8, 0.99), (10, 0.1), (8, 0.5)])
def test_draft_gate_fanouts(f0, rho):
    d = I.make_verify_batch(2, 7, 3 * 8192, I.BF16, seed=f0)
    m, g, c = _run(d["zd"], d["tok"], I.BF16, f0, rho, 0.5)
    _check(d["zd"], d["tok"], I.BF16, f0, rho, 0.5, m, g, c)


def test_draft_gate_margin_only():
    d = I.make_verify_batch(4, 3, 8192 + 4096, I.BF16, seed=3)
    m, g, c = _run(d["zd"], d["tok"], I.BF16, 0, 0.5, 0.4)
    assert c is None
    for s in range(4):
        o = DO.draft_pass(I.as_f64(d["zd"][s], I.BF16), d["tok"][s], 0, 0.5, float(np.float32(0.4)))
        assert np.all(np.abs(m[s] - o["margin"]) <= 1e-5 * o["margin"] + 2e-6) and np.array_equal(g[s], o["gate"])


def test_draft_gate_many_equal_logits_and_masked_words():
    """Logits quantised to steps of 0.5 (hundreds of ties at every level: the threshold list overflows and the
    block-wide rounds take over), a masked tail, an all-equal row, drafted tokens at the top / outside the top /
    outside the vocabulary."""
    dtype, V = I.FP32, 2 * 8192 + 1024
    rng = np.random.default_rng(17)
    zd = (np.round(rng.standard_normal((2, 4, V)) * 4) / 2).astype(np.float32)
    zd[:, :, V - 700:] = -np.inf
    zd[1, 2, :] = 1.25                                  # all equal: margin 0, candidates 0, 1, 2, ... skipping the token
    zd[1, 3, :] = -np.inf
    zd[1, 3, 100:110] = 0.0                             # ten live words only: fewer candidates than asked for
    tok = np.argmax(zd, axis=2).astype(np.int32)        # the top word (first among equals)
    tok[0, 1] = 5                                       # outside the top
    tok[0, 2] = -1                                      # outside the vocabulary: excludes nothing
    tok[0, 3] = V + 7
    tok[1, 2] = 3
    tok[1, 3] = 104
    f0 = 12
    m, g, c = _run(zd, tok, dtype, f0, 0.999, 0.05)
    assert m[1, 2] == 0.0 and list(c[1, 2]) == [0, 1, 2, 4, 5, 6, 7, 8, 9, 10, 11, 12]
    # ten live words, one of them drafted: nine finite candidates, then masked words in index order
    assert list(c[1, 3][:9]) == [100, 101, 102, 103, 105, 106, 107, 108, 109] and list(c[1, 3][9:]) == [0, 1, 2]
    _check(zd, tok, dtype, f0, 0.999, 0.05, m, g, c)


def test_draft_gate_full_vocabulary_batch():
    """The benchmark's shape (64 x 8 positions over 151,936 words, bf16); every fourth sequence against the oracle."""
    dtype = I.BF16
    d = I.make_verify_batch(64, 8, I.VERIFY_VOCAB, dtype, seed=2024)
    m, g, c = _run(d["zd"], d["tok"], dtype, 8, 0.5, 0.5)
    assert 0 < g.sum() < g.size                          # both gate outcomes occur
    _check(d["zd"], d["tok"], dtype, 8, 0.5, 0.5, m, g, c, seqs=range(0, 64, 4))
