"""Pins of oracle/draft_oracle.py against what the paper's equations and the mathematics fix (Sec. III-B
margin and gating equations, Sec. III-C fan-out equation and candidate rule).  CPU only."""
import math

import numpy as np
import pytest

from oracle import draft_oracle as DO


def test_margin_two_words_is_tanh_of_half_the_gap():
    for a, b in [(0.3, -1.2), (5.0, 5.0), (-2.0, 3.5), (100.0, 99.0)]:
        assert DO.margin(np.array([a, b])) == pytest.approx(math.tanh(abs(a - b) / 2), rel=1e-12, abs=1e-15)


def test_margin_one_boosted_word_closed_form():
    V, delta = 1000, 3.0
    z = np.full(V, -0.7)
    z[417] += delta
    want = (math.exp(delta) - 1.0) / (math.exp(delta) + V - 1)
    assert DO.margin(z) == pytest.approx(want, rel=1e-12)
    # a common shift of all logits changes nothing; a runner-up halves the gap to the top
    assert DO.margin(z + 55.0) == pytest.approx(want, rel=1e-12)
    z[3] += delta
    assert DO.margin(z) == pytest.approx(0.0, abs=1e-15)


def test_margin_uses_the_two_largest_not_the_first_two():
    z = np.array([0.0, 0.1, 4.0, -3.0, 3.0])
    p = np.exp(z) / np.exp(z).sum()
    assert DO.margin(z) == pytest.approx(p[2] - p[4], rel=1e-13)


def test_gate_commits_at_and_above_the_threshold():
    assert DO.gate(0.5, 0.5) == 0 and DO.gate(0.6, 0.5) == 0 and DO.gate(0.4, 0.5) == 1
    assert DO.gate(0.0, 0.0) == 0
    # decided in float32: a margin that rounds onto gamma commits
    assert DO.gate(0.5 - 1e-12, 0.5) == 0


def test_fanout_sequence():
    assert DO.fanout(8, 0.5, 6) == [8, 4, 2, 1, 1, 1]         # ceil(8 * 2^-j); never below one
    assert DO.fanout(5, 0.6, 4) == [5, 3, 2, 2]               # 5, 3.0, 1.8, 1.08
    assert DO.fanout(1, 0.9, 3) == [1, 1, 1]
    # decimal rho whose products are exact integers in the fan-out equation: binary rounding of rho or of the power
    # must not tip them over (10 * 0.1 = 1, 30 * 0.1 = 3, 20 * 0.3^2 = 1.8, 100 * 0.7^2 = 49)
    assert DO.fanout(10, 0.1, 3) == [10, 1, 1]
    assert DO.fanout(30, 0.1, 3) == [30, 3, 1]
    assert DO.fanout(20, 0.3, 3) == [20, 6, 2]
    assert DO.fanout(100, 0.7, 3) == [100, 70, 49]
    f = DO.fanout(16, 0.7, 12)
    assert f[0] == 16 and all(a >= b >= 1 for a, b in zip(f, f[1:]))


def test_candidates_match_repeated_argmax_without_the_drafted_token():
    rng = np.random.default_rng(3)
    for trial in range(20):
        V = int(rng.integers(5, 60))
        z = np.round(rng.standard_normal(V) * 2, 1)             # rounded: ties occur
        y = int(rng.integers(0, V))
        f = int(rng.integers(1, 6))
        got = DO.candidates(z, y, f)
        zz = z.copy()
        zz[y] = -np.inf
        want = []
        for _ in range(min(f, V - 1)):
            w = int(np.argmax(zz))                               # first index among equals
            want.append(w)
            zz[w] = -np.inf
        assert list(got) == want
        assert y not in got and len(set(got.tolist())) == len(got)
        rest = np.setdiff1d(np.arange(V), np.append(got, y))
        if len(rest) and len(got):
            assert z[rest].max() <= z[got].min()


def test_candidates_when_the_drafted_token_is_the_top_word_or_not_in_the_top():
    z = np.array([1.0, 9.0, 3.0, 7.0, 5.0])
    assert list(DO.candidates(z, 1, 2)) == [3, 4]               # top word drafted: the next two
    assert list(DO.candidates(z, 0, 2)) == [1, 3]               # drafted word outside the top: plain top-2
    assert list(DO.candidates(z, 3, 10)) == [1, 4, 2, 0]        # fewer other words than asked for


def test_draft_pass_shapes_and_consistency():
    rng = np.random.default_rng(0)
    zd = rng.standard_normal((5, 40)) * 3
    tok = zd.argmax(axis=1)
    out = DO.draft_pass(zd, tok, f0=4, rho=0.5, gamma=0.3)
    assert out["fanout"] == [4, 2, 1, 1, 1]
    assert [len(c) for c in out["cand"]] == out["fanout"]
    for t in range(5):
        assert tok[t] not in out["cand"][t]
        assert out["gate"][t] == (0 if np.float32(out["margin"][t]) >= np.float32(0.3) else 1)
        # the drafted word is the top word here, so the first candidate is the runner-up of the margin
        p = np.exp(zd[t] - zd[t].max())
        p /= p.sum()
        assert out["margin"][t] == pytest.approx(p[tok[t]] - p[out["cand"][t][0]], rel=1e-12)
