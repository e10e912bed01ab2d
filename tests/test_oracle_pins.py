"""Pins for the CPU oracle: closed forms, invariants, textbook routines, brute force.

Each test names the passage of the paper (Section III-A) whose statement it
pins.  None of the expected values comes from the oracle itself or from the
GPU path: they are closed forms, SciPy routines that are not used inside the
oracle, or exhaustive enumeration.
"""
import itertools

import numpy as np
import pytest
import scipy.linalg
import scipy.spatial.distance
import scipy.special

from oracle import covspec_oracle as O

rng0 = np.random.default_rng(7)


def _rand(*shape, rng=None):
    return (rng or rng0).standard_normal(shape)


# ---------------------------------------------------------------- embeddings
def test_embed_is_row_vector_times_in_by_out_weight():
    # W[i, (i+1) % d] = 1 moves component i to position i+1; a transposed
    # operand would move it the other way.
    d = 6
    W = np.zeros((d, d))
    W[np.arange(d), (np.arange(d) + 1) % d] = 1.0
    x = np.arange(1.0, d + 1)[None, :]
    np.testing.assert_array_equal(O.embed(x, W), np.roll(x, 1, axis=1))
    assert O.embed(x, None) is not None and np.array_equal(O.embed(x, None), x)


# ---------------------------------------------------------------- query score (cosine-max equation)
def test_cosine_single_keyword_matches_scipy():
    X, q = _rand(9, 5), _rand(1, 5)
    ref = np.array([1.0 - scipy.spatial.distance.cosine(x, q[0]) for x in X])
    np.testing.assert_allclose(O.query_score_cosine(X, q), ref, rtol=0, atol=1e-14)


def test_cosine_is_max_over_keywords_not_mean_or_min():
    X, Q = _rand(7, 4), _rand(3, 4)
    ref = np.array([max(1.0 - scipy.spatial.distance.cosine(x, q) for q in Q) for x in X])
    np.testing.assert_allclose(O.query_score_cosine(X, Q), ref, atol=1e-14)


def test_cosine_parallel_antiparallel_and_range():
    q = _rand(1, 8)
    X = np.vstack([2.5 * q, -0.3 * q, _rand(4, 8)])
    s = O.query_score_cosine(X, q)
    assert abs(s[0] - 1.0) < 1e-15 and abs(s[1] + 1.0) < 1e-15
    assert np.all(s <= 1 + 1e-15) and np.all(s >= -1 - 1e-15)


def test_cosine_invariances():
    X, Q = _rand(20, 6), _rand(4, 6)
    base = O.query_score_cosine(X, Q)
    scale = np.exp(_rand(20))[:, None]           # positive token rescale (norm outliers)
    np.testing.assert_allclose(O.query_score_cosine(X * scale, Q), base, atol=1e-14)
    np.testing.assert_allclose(O.query_score_cosine(X, Q * np.array([[3.0], [0.1], [7.0], [1.0]])), base, atol=1e-14)
    np.testing.assert_allclose(O.query_score_cosine(X, Q[[2, 0, 3, 1]]), base, atol=0)
    R, _ = np.linalg.qr(_rand(6, 6))             # same orthogonal map on both sides
    via = O.query_score_cosine(O.embed(X, R), O.embed(Q, R))
    np.testing.assert_allclose(via, base, atol=1e-13)


def test_cosine_uses_separate_weights_for_tokens_and_keywords():
    # Wk shifts components right, Wq is identity: cos(shift(x), q).
    d = 5
    Wk = np.zeros((d, d)); Wk[np.arange(d), (np.arange(d) + 1) % d] = 1.0
    X, Q = _rand(6, d), _rand(2, d)
    got = O.score(X, None, Q, None, Wk, O.Params())["s_query"]
    ref = np.array([max(1.0 - scipy.spatial.distance.cosine(np.roll(x, 1), q) for q in Q) for x in X])
    np.testing.assert_allclose(got, ref, atol=1e-14)
    got2 = O.score(X, None, Q, Wk, None, O.Params())["s_query"]
    ref2 = np.array([max(1.0 - scipy.spatial.distance.cosine(x, np.roll(q, 1)) for q in Q) for x in X])
    np.testing.assert_allclose(got2, ref2, atol=1e-14)


def test_cosine_zero_vector_scores_zero():
    X = np.vstack([np.zeros(4), _rand(2, 4)])
    assert O.query_score_cosine(X, _rand(2, 4))[0] == 0.0


# ---------------------------------------------------------------- attention variant
def test_attention_rows_sum_to_one_and_total_mass():
    Ev, Eq = _rand(33, 12), _rand(5, 12)
    A = O.attention_rows(Ev, Eq, 3)
    assert A.shape == (3, 5, 33) and np.all(A >= 0)
    np.testing.assert_allclose(A.sum(axis=2), 1.0, atol=1e-14)
    assert abs(O.query_score_attention(Ev, Eq, 3).sum() - 1.0) < 1e-13


def test_attention_single_head_single_query_is_textbook_softmax():
    Ev, Eq = _rand(17, 8), _rand(1, 8)
    ref = scipy.special.softmax(Ev @ Eq[0] / np.sqrt(8.0))
    np.testing.assert_allclose(O.query_score_attention(Ev, Eq, 1), ref, atol=1e-15)


def test_attention_zero_query_uniform_and_shift_invariance():
    Ev = _rand(10, 8)
    np.testing.assert_allclose(O.query_score_attention(Ev, np.zeros((3, 8)), 2), 0.1, atol=1e-15)
    Eq = _rand(3, 8)
    u = _rand(1, 8)                               # adds the constant Eq_j.u to every logit of a row
    np.testing.assert_allclose(O.query_score_attention(Ev + u, Eq, 2),
                               O.query_score_attention(Ev, Eq, 2), atol=1e-13)


def test_attention_heads_are_column_blocks_with_sqrt_dh_scale():
    # query mass only in head 0's columns: head 1 is uniform, head 0 is a softmax over dh=4 dims.
    Ev, Eq = _rand(9, 8), _rand(1, 8)
    Eq[:, 4:] = 0.0
    ref = 0.5 * scipy.special.softmax(Ev[:, :4] @ Eq[0, :4] / 2.0) + 0.5 / 9
    np.testing.assert_allclose(O.query_score_attention(Ev, Eq, 2), ref, atol=1e-15)


# ---------------------------------------------------------------- activity score equation
def test_activity_closed_forms():
    N, d, K = 6, 5, 3
    H0 = _rand(N, d)
    assert np.all(O.activity_score(np.stack([H0] * (K + 1))) == 0.0)
    u = _rand(d); u /= np.linalg.norm(u)
    a = np.array([0.5, -2.0, 1.25])
    Hs = [H0]
    for al in a:
        Hs.append(Hs[-1] + al * u)
    np.testing.assert_allclose(O.activity_score(np.stack(Hs)), np.mean(np.abs(a)), atol=1e-14)
    # 3-4-5 triangle, K = 1
    Hs = np.zeros((2, 1, 2)); Hs[1, 0] = (3.0, 4.0)
    assert O.activity_score(Hs)[0] == 5.0


def test_activity_k1_is_euclidean_distance_and_degree_one():
    A, B = _rand(8, 7), _rand(8, 7)
    ref = np.array([scipy.spatial.distance.euclidean(a, b) for a, b in zip(A, B)])
    got = O.activity_score(np.stack([A, B]))
    np.testing.assert_allclose(got, ref, atol=1e-14)
    np.testing.assert_allclose(O.activity_score(3.5 * np.stack([A, B])), 3.5 * ref, atol=1e-13)
    assert np.all(got >= 0)


def test_activity_is_mean_of_norms_not_norm_of_mean():
    # two steps that cancel: the telescoped difference is zero but the activity is not
    H0 = np.zeros((1, 3)); H1 = np.array([[1.0, 0, 0]])
    assert O.activity_score(np.stack([H0, H1, H0]))[0] == 1.0


# ---------------------------------------------------------------- fusion equation
def test_minmax_and_fuse_worked_example():
    sq, sa = np.array([1.0, 2.0, 3.0]), np.array([10.0, 30.0, 20.0])
    np.testing.assert_allclose(O.fuse(sq, sa, 0.25), [0.0, 0.875, 0.625], atol=1e-15)
    m = O.minmax(_rand(50))
    assert m.min() == 0.0 and m.max() == 1.0
    assert np.all(O.minmax(np.full(5, 3.3)) == 0.0)


def test_fuse_limits_and_affine_invariance():
    sq, sa = _rand(40), np.abs(_rand(40))
    np.testing.assert_array_equal(np.argsort(-O.fuse(sq, sa, 1.0), kind="stable"), np.argsort(-sq, kind="stable"))
    np.testing.assert_array_equal(np.argsort(-O.fuse(sq, sa, 0.0), kind="stable"), np.argsort(-sa, kind="stable"))
    np.testing.assert_allclose(O.fuse(4.0 * sq - 9.0, 0.5 * sa + 2.0, 0.3), O.fuse(sq, sa, 0.3), atol=1e-14)
    np.testing.assert_allclose(O.fuse(sq, None, 0.3), O.minmax(sq), atol=0)


# ---------------------------------------------------------------- ranking decisions
def test_top_indices_ties_go_to_lower_index_and_output_ascending():
    s = np.array([0.5, 0.9, 0.5, 0.9, 0.1, 0.5])
    np.testing.assert_array_equal(O.top_indices(s, 3), [0, 1, 3])
    np.testing.assert_array_equal(O.top_indices(s, 4), [0, 1, 2, 3])
    np.testing.assert_array_equal(O.top_indices(s, 6), np.arange(6))
    # values that differ only below float32 resolution are ties for the decision
    s = np.array([1.0, 1.0 + 1e-12, 0.0])
    np.testing.assert_array_equal(O.top_indices(s, 1), [0])


@pytest.mark.parametrize("n,k", [(6, 2), (8, 3), (10, 4), (9, 9)])
def test_topk_equals_exhaustive_subset_optimum(n, k):
    # the paper's criterion "retain the k largest energies" maximises sum_{i in S} c_i over |S| = k
    rng = np.random.default_rng(n * 100 + k)
    c = rng.integers(0, 5, size=n).astype(np.float64)      # many ties on purpose
    best, best_set = -1.0, None
    for S in itertools.combinations(range(n), k):           # lexicographic order: first maximum wins
        v = c[list(S)].sum()
        if v > best:
            best, best_set = v, S
    got = O.top_indices(c, k)
    assert c[got].sum() == best
    np.testing.assert_array_equal(got, best_set)
    assert len(set(got.tolist())) == k and np.all(np.diff(got) > 0)


def test_top_indices_permutation_equivariance():
    s = _rand(30)
    perm = np.random.default_rng(3).permutation(30)
    a = set(perm[O.top_indices(s[perm], 7)].tolist())
    assert a == set(O.top_indices(s, 7).tolist())


def test_cut_margin():
    s = np.array([4.0, 1.0, 3.0, 2.0])
    assert O.cut_margin(s, 2) == pytest.approx(0.25)
    assert O.cut_margin(s, 4) == float("inf")


# ---------------------------------------------------------------- low-rank energy (SVD / energy equations)
def test_energy_diagonal_closed_form():
    s = np.array([3.0, 0.5, 2.0, 1.0])
    Z = np.diag(s)                                         # z_i = s_i e_i
    c, sig = O.subspace_energy(Z, 2)
    np.testing.assert_allclose(sig, [3, 2, 1, 0.5], atol=1e-15)
    np.testing.assert_allclose(c, [9.0, 0.0, 4.0, 0.0], atol=1e-14)


def test_energy_sums_bounds_and_eckart_young():
    Z = _rand(14, 9)
    r = 4
    c, _ = O.subspace_energy(Z, r)
    lam = scipy.linalg.eigh(Z @ Z.T, eigvals_only=True)[::-1]       # independent routine
    assert c.sum() == pytest.approx(lam[:r].sum(), rel=1e-12)
    n2 = np.sum(Z * Z, axis=1)
    assert np.all(c >= -1e-13) and np.all(c <= n2 + 1e-12)
    assert (n2 - c).sum() == pytest.approx(lam[r:].sum(), rel=1e-11)  # = ||Z - Z_r||_F^2


def test_energy_equals_projection_on_left_subspace_from_the_other_gram():
    # c_i = ||U_r^T z_i||^2 with U_r from the d x d matrix Z_M Z_M^T
    Z = _rand(12, 7)
    r = 3
    w, U = scipy.linalg.eigh(Z.T @ Z)
    Ur = U[:, ::-1][:, :r]
    ref = np.sum((Z @ Ur) ** 2, axis=1)
    np.testing.assert_allclose(O.subspace_energy(Z, r)[0], ref, atol=1e-12)
    # wide case (M > d route)
    Z = _rand(6, 11)
    w, U = scipy.linalg.eigh(Z.T @ Z)
    ref = np.sum((Z @ U[:, ::-1][:, :2]) ** 2, axis=1)
    np.testing.assert_allclose(O.subspace_energy(Z, 2)[0], ref, atol=1e-12)


def test_energy_rank1_power_iteration_exact_rank_rotation_and_duplicates():
    Z = _rand(10, 6)
    u = np.ones(6)
    for _ in range(2000):
        u = Z.T @ (Z @ u); u /= np.linalg.norm(u)
    np.testing.assert_allclose(O.subspace_energy(Z, 1)[0], (Z @ u) ** 2, atol=1e-10)
    Zr = _rand(10, 3) @ _rand(3, 6)                        # exact rank 3
    np.testing.assert_allclose(O.subspace_energy(Zr, 3)[0], np.sum(Zr * Zr, axis=1), rtol=1e-12)
    R, _ = np.linalg.qr(_rand(6, 6))
    np.testing.assert_allclose(O.subspace_energy(Z @ R, 2)[0], O.subspace_energy(Z, 2)[0], atol=1e-12)
    Zd = Z.copy(); Zd[7] = Zd[2]
    c = O.subspace_energy(Zd, 3)[0]
    assert abs(c[7] - c[2]) < 1e-13 * c[2]


def test_energy_no_mean_centering():
    # a common offset is part of the representation: c changes if it were removed
    Z = _rand(8, 5) + 10.0
    c, sig = O.subspace_energy(Z, 1)
    assert sig[0] ** 2 > 0.9 * np.sum(Z * Z)


# ---------------------------------------------------------------- greedy variant
def _ls_residual(Z, S, i):
    if not S:
        return float(Z[i] @ Z[i])
    A = Z[list(S)].T
    coef, *_ = np.linalg.lstsq(A, Z[i], rcond=None)
    e = Z[i] - A @ coef
    return float(e @ e)


def test_greedy_each_pick_has_largest_least_squares_residual():
    Z = _rand(9, 6)
    order, resid = O.greedy_residual(Z, 5)
    assert order[0] == np.argmax(np.sum(Z * Z, axis=1))
    S = []
    for t, p in enumerate(order):
        res = np.array([_ls_residual(Z, S, i) if i not in S else -1.0 for i in range(9)])
        assert p == np.argmax(res)
        assert resid[t] == pytest.approx(res[p], rel=1e-10)
        S.append(int(p))
    assert np.all(np.diff(resid) <= 1e-12)
    G = Z @ Z.T
    assert np.prod(resid) == pytest.approx(np.linalg.det(G[np.ix_(order, order)]), rel=1e-10)


def test_greedy_matches_column_pivoted_qr():
    Z = _rand(12, 8)
    _, _, piv = scipy.linalg.qr(Z.T, pivoting=True)
    order, _ = O.greedy_residual(Z, 6)
    np.testing.assert_array_equal(order, piv[:6])


def test_greedy_exact_rank_leaves_no_residual_and_skips_duplicates():
    Z = _rand(12, 3) @ _rand(3, 7)
    Z[9] = Z[4]
    order, resid = O.greedy_residual(Z, 5)
    tr = np.sum(Z * Z)
    assert np.all(resid[3:] <= 1e-10 * tr)
    first3 = set(order[:3].tolist())
    assert not {4, 9} <= first3
    # full-rank case with a duplicate: never both among picks made while residual is non-zero
    Z = _rand(10, 8); Z[6] = Z[1]
    order, resid = O.greedy_residual(Z, 8)
    live = [int(p) for p, r_ in zip(order, resid) if r_ > 1e-9]
    assert not {1, 6} <= set(live)
    assert 1 in live and 6 not in live                     # tie on the first encounter -> lower index


# ---------------------------------------------------------------- whole path
def test_select_contracts_and_identity_case():
    X, s = _rand(20, 6), _rand(20)
    p = O.Params(keep_k=4, preselect_m=8, rank_r=2)
    out = O.select(X, s, p)
    assert out["idx_m"].shape == (8,) and out["idx"].shape == (4,)
    assert set(out["idx"].tolist()) <= set(out["idx_m"].tolist())
    assert np.all(np.diff(out["idx"]) > 0) and out["idx"].dtype == np.int32
    for mode in (0, 1):
        full = O.select(X, s, O.Params(keep_k=20, preselect_m=20, rank_r=2, lr_mode=mode))
        np.testing.assert_array_equal(full["idx"], np.arange(20))


def test_params_defaults():
    p = O.Params(keep_ratio=0.1)
    assert p.resolved(8192) == (819, 1638, 409)
    assert O.Params(keep_k=64).resolved(576) == (64, 128, 32)
    assert O.Params(keep_k=400).resolved(576) == (400, 576, 200)


def test_reduce_gathers_stored_rows_and_is_deterministic():
    rng = np.random.default_rng(11)
    X, Q, Hs = rng.standard_normal((30, 8)), rng.standard_normal((3, 8)), rng.standard_normal((3, 30, 8))
    W = rng.standard_normal((8, 8))
    p = O.Params(keep_k=5, preselect_m=10, rank_r=3, lam=0.4)
    a = O.reduce(X, Hs, Q, W, W.T.copy(), p)
    b = O.reduce(X, Hs, Q, W, W.T.copy(), p)
    np.testing.assert_array_equal(a["idx"], b["idx"])
    np.testing.assert_array_equal(a["tokens"], X[a["idx"]])
    assert a["tokens"].shape == (5, 8)


def test_low_rank_stage_uses_raw_features_not_embeddings():
    # scaling Wk changes no cosine, so the kept set must not move; scaling X rows moves energies
    rng = np.random.default_rng(12)
    X, Q = rng.standard_normal((16, 6)), rng.standard_normal((2, 6))
    Wk = rng.standard_normal((6, 6))
    p = O.Params(keep_k=3, preselect_m=16, rank_r=2, lam=1.0)
    a = O.reduce(X, None, Q, None, Wk, p)
    b = O.reduce(X, None, Q, None, 5.0 * Wk, p)
    np.testing.assert_array_equal(a["idx"], b["idx"])
    np.testing.assert_allclose(a["c"], b["c"], rtol=1e-12)


# --------------------------------------------------------------------------
# selector ablations (Table II rows "full-token" / "random-token"; Sec. III-A.3 "the M highest-scoring tokens")
# --------------------------------------------------------------------------
def test_mix64_reproduces_the_published_splitmix64_outputs():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "splitmix64_seed0.txt")
    want = [int(l, 16) for l in open(path) if l.strip() and not l.startswith("#")]
    gamma = 0x9E3779B97F4A7C15
    got = [O.mix64(((i + 1) * gamma) & ((1 << 64) - 1)) for i in range(len(want))]
    assert got == want


def test_random_scores_are_24_bit_uniforms_keyed_by_seed_image_and_token():
    u = O.random_scores(3, 5, 4096)
    assert np.all((u >= 0) & (u < 1)) and np.all(u * 2 ** 24 == np.floor(u * 2 ** 24))
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)          # exact in float32
    # the word construction, restated: seed * gamma + (image << 32 | token) + constant, top 24 bits of the mix
    word = (3 * 0x9E3779B97F4A7C15 + ((5 << 32) | 17) + 0x632BE59BD9B4E019) % (1 << 64)
    assert u[17] == (O.mix64(word) >> 40) / 2.0 ** 24
    # different seed / image / token give different streams; same arguments give the same stream
    assert np.array_equal(u, O.random_scores(3, 5, 4096))
    assert not np.array_equal(u, O.random_scores(4, 5, 4096)) and not np.array_equal(u, O.random_scores(3, 6, 4096))
    # uniformity: mean and variance of U(0,1), and a coarse chi-square over 16 bins (dof 15, 99.9 % point 37.7)
    big = O.random_scores(11, 0, 1 << 16)
    assert abs(big.mean() - 0.5) < 5e-3 and abs(big.var() - 1 / 12) < 2e-3
    counts = np.bincount((big * 16).astype(int), minlength=16)
    assert ((counts - 4096.0) ** 2 / 4096.0).sum() < 37.7


def test_random_selection_is_a_uniform_draw_without_replacement():
    rng = np.random.default_rng(5)
    X = rng.standard_normal((64, 8))
    hits = np.zeros(64)
    for seed in range(400):
        out = O.select(X, None, O.Params(lr_mode=O.LR_RANDOM, keep_k=16, preselect_m=32, seed=seed), image=2)
        idx = out["idx"]
        assert idx.dtype == np.int32 and len(idx) == 16 and np.all(np.diff(idx) > 0)
        assert np.array_equal(idx, O.top_indices(O.random_scores(seed, 2, 64), 16))
        hits[idx] += 1
    # every token is kept with probability k/N = 1/4: 400 draws -> mean 100, sd 8.7
    assert abs(hits.mean() - 100) < 1e-9 and hits.min() > 60 and hits.max() < 140


def test_score_only_selection_keeps_the_k_highest_fused_scores():
    rng = np.random.default_rng(6)
    X = rng.standard_normal((50, 6))
    s = rng.standard_normal(50)
    out = O.select(X, s, O.Params(lr_mode=O.LR_SCORE_TOPK, keep_k=7, preselect_m=20))
    assert set(out["idx"]) == set(np.argsort(-s, kind="stable")[:7]) and np.all(np.diff(out["idx"]) > 0)
    assert set(out["idx"]) <= set(out["idx_m"]) and len(out["idx_m"]) == 20
    # the low-rank modes may keep different tokens from the same pre-selection
    full = O.select(X, s, O.Params(lr_mode=O.LR_ENERGY_TOPK, keep_k=7, preselect_m=20, rank_r=3))
    assert set(full["idx"]) <= set(out["idx_m"])
