"""Pins of the verification oracle against what the paper (Sec. II-A) and the mathematics fix."""
import itertools

import numpy as np
import pytest
import scipy.special

from oracle import verify_oracle as V


def test_softmax_matches_scipy_and_is_shift_invariant():
    rng = np.random.default_rng(1)
    z = rng.standard_normal((5, 37)) * 4
    np.testing.assert_allclose(V.softmax(z), scipy.special.softmax(z, axis=-1), rtol=1e-14, atol=0)
    np.testing.assert_allclose(V.softmax(z + 1000.0), V.softmax(z), rtol=1e-12)        # no overflow, same result
    np.testing.assert_allclose(V.softmax(z).sum(axis=-1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(V.softmax(np.zeros(8)), np.full(8, 1 / 8))


def test_acceptance_probability_closed_forms():
    pt = np.array([0.5, 0.3, 0.2])
    pd = np.array([0.25, 0.6, 0.15])
    assert V.accept_prob(pt, pd, 0) == 1.0            # target likes it more: always accepted
    assert V.accept_prob(pt, pd, 1) == pytest.approx(0.5)
    assert V.accept_prob(pt, pd, 2) == 1.0
    assert V.accept_prob(pt, pt, 1) == 1.0            # identical models never reject
    assert V.accept_prob(pt, np.array([1.0, 0.0, 0.0]), 1) == 1.0


def test_residual_is_a_distribution_supported_where_target_exceeds_draft():
    rng = np.random.default_rng(2)
    pt, pd = V.softmax(rng.standard_normal(50) * 2), V.softmax(rng.standard_normal(50) * 2)
    w = V.residual_weights(pt, pd)
    assert np.all(w >= 0) and np.all((w > 0) == (pt > pd))
    # total residual mass = 1 - sum_w min(p_t, p_d) = total variation distance = rejection probability
    assert w.sum() == pytest.approx(1.0 - np.minimum(pt, pd).sum(), rel=1e-12)
    assert w.sum() == pytest.approx(0.5 * np.abs(pt - pd).sum(), rel=1e-12)


def test_accept_or_resample_reproduces_the_target_distribution_exactly():
    # the identity speculative sampling rests on: P(out = w) = p_d(w) alpha(w) + P(reject) r(w) = p_t(w)
    rng = np.random.default_rng(3)
    for _ in range(5):
        pt, pd = V.softmax(rng.standard_normal(23) * 3), V.softmax(rng.standard_normal(23) * 3)
        alpha = np.array([V.accept_prob(pt, pd, w) for w in range(23)])
        w = V.residual_weights(pt, pd)
        p_reject = 1.0 - (pd * alpha).sum()
        out = pd * alpha + p_reject * w / w.sum()
        np.testing.assert_allclose(out, pt, rtol=1e-12, atol=1e-15)


def test_inverse_cdf_brute_force_and_boundaries():
    w = np.array([0.0, 2.0, 0.0, 1.0, 1.0])
    # cumulative: 0 2 2 3 4 ; target = u * 4
    assert V.inverse_cdf(w, 0.0) == 1                 # skips the zero-weight head
    assert V.inverse_cdf(w, 0.49) == 1
    assert V.inverse_cdf(w, 0.5) == 3                 # target equals a CDF step: strictly greater is required
    assert V.inverse_cdf(w, 0.74) == 3
    assert V.inverse_cdf(w, 0.75) == 4
    assert V.inverse_cdf(w, 0.999999) == 4
    rng = np.random.default_rng(4)
    ww = rng.random(200) * (rng.random(200) > 0.5)
    for u in rng.random(100):
        c, tgt = 0.0, u * np.cumsum(ww)[-1]
        for i, x in enumerate(ww):                    # the definition, written out
            c += x
            if c > tgt:
                break
        assert V.inverse_cdf(ww, u) == i
    # draws follow the weights: 20000 stratified uniforms
    counts = np.bincount([V.inverse_cdf(w, (j + 0.5) / 20000) for j in range(20000)], minlength=5)
    np.testing.assert_allclose(counts / 20000, w / w.sum(), atol=1e-4)


def test_verify_stops_at_the_first_rejection():
    rng = np.random.default_rng(5)
    L, Vn = 6, 40
    zt = rng.standard_normal((L, Vn)) * 2
    zd = zt + rng.standard_normal((L, Vn))
    tok = rng.integers(0, Vn, L)
    pt, pd = V.softmax(zt), V.softmax(zd)
    alpha = np.array([min(1.0, pt[t, tok[t]] / pd[t, tok[t]]) for t in range(L)])
    # uniforms chosen around alpha: accept the first three, reject the fourth, later ones irrelevant
    u = np.array([0.0, alpha[1] * 0.5, alpha[2] * 0.999, 1.0 - 1e-7, 0.0, 0.0], dtype=np.float32)
    if alpha[3] == 1.0:
        tok[3] = int(np.argmax(pd[3] - pt[3]))        # a token the draft over-weights
    out = V.verify(zt, zd, tok, u, 0.3)
    assert out["n_acc"] == 3 and 0 <= out["corr"] < Vn
    assert pt[3, out["corr"]] > pd[3, out["corr"]]    # corrections come from the residual's support
    assert out["corr"] == V.inverse_cdf(np.maximum(pt[3] - pd[3], 0), 0.3)
    np.testing.assert_allclose(out["alpha"][:3], alpha[:3], rtol=1e-12)
    # everything accepted: no correction
    out = V.verify(zt, zt, tok, np.full(L, 0.999999, dtype=np.float32), 0.5)
    assert out["n_acc"] == L and out["corr"] == -1 and np.all(out["alpha"] == 1.0)
    # a uniform of exactly 1 (outside [0, 1)) forces a rejection although the models agree: the residual has
    # no mass, and the correction falls back to argmax p_t
    out = V.verify(zt[:1], zt[:1], tok[:1], np.array([1.0], dtype=np.float32), 0.5)
    assert out["n_acc"] == 0 and out["residual_mass"] == 0.0 and out["corr"] == int(np.argmax(pt[0]))


def test_verify_exhaustive_on_a_two_word_vocabulary():
    # V = 2, one position: p_t = (a, 1-a), p_d = (b, 1-b); drafted word 0
    for a, b in itertools.product([0.2, 0.5, 0.9], [0.3, 0.5, 0.8]):
        zt = np.log(np.array([[a, 1 - a]])); zd = np.log(np.array([[b, 1 - b]]))
        for u in [0.0, 0.3, 0.6, 0.99]:
            out = V.verify(zt, zd, np.array([0]), np.array([u], dtype=np.float32), 0.5)
            al = min(1.0, a / b)
            assert out["alpha"][0] == pytest.approx(al, rel=1e-12)
            if np.float32(u) < np.float32(al):
                assert out["n_acc"] == 1 and out["corr"] == -1
            else:
                assert out["n_acc"] == 0 and out["corr"] == 1      # rejection of word 0 means b > a: residual on word 1
