"""Pins of oracle/stream_oracle.py: the frame-by-frame composition of the pinned selection steps."""
import numpy as np
import pytest

from oracle import covspec_oracle as O
from oracle import stream_oracle as S


def _frames(n_frames, n_f, d, seed, rank=None):
    rng = np.random.default_rng(seed)
    rank = rank or d
    basis = rng.standard_normal((rank, d))
    decay = np.exp(-0.15 * np.arange(rank))
    X = [(rng.standard_normal((n_f, rank)) * decay) @ basis for _ in range(n_frames)]
    s = [rng.random(n_f) for _ in range(n_frames)]
    return X, s


def test_everything_is_kept_while_the_memory_is_not_full():
    # k at least the number of pre-selected tokens seen so far: the state is the pre-selected tokens of every frame,
    # in arrival order, and no energy is computed
    X, s = _frames(3, 20, 8, 0)
    st = S.empty_state(8)
    for f in range(3):
        out = S.stream_step(st, X[f], s[f], id_base=100 * f, frame_m=5, keep_k=15, rank_r=2)
        assert out["c"] is None
    want = np.concatenate([100 * f + O.top_indices(s[f], 5) for f in range(3)])
    np.testing.assert_array_equal(st.ids, want)
    np.testing.assert_array_equal(st.rows, np.concatenate([X[f][O.top_indices(s[f], 5)] for f in range(3)]))


def test_first_frame_is_the_one_image_selection_of_the_paper():
    # empty memory and M_f > k: the step is Sec. III-A.3 on one image (pre-select M, energy, keep k)
    X, s = _frames(1, 60, 16, 1)
    st = S.empty_state(16)
    out = S.stream_step(st, X[0], s[0], id_base=0, frame_m=24, keep_k=10, rank_r=4)
    ref = O.select(X[0], s[0], O.Params(preselect_m=24, rank_r=4, keep_k=10))
    np.testing.assert_array_equal(st.ids, ref["idx"])
    np.testing.assert_allclose(out["c"], ref["c"], rtol=1e-12)


def test_energies_are_the_diagonal_of_the_best_rank_r_approximation_of_the_candidate_gram_matrix():
    # independent route: eigen-decomposition of the candidates' Gram matrix assembled from the CARRIED block and the
    # new rows (the shortcut the library takes), instead of the SVD of the stacked rows
    X, s = _frames(4, 30, 12, 2)
    st = S.empty_state(12)
    k, m, r = 14, 9, 3
    G_keep = np.zeros((0, 0))
    for f in range(4):
        kept_rows = st.rows.copy()
        out = S.stream_step(st, X[f], s[f], id_base=30 * f, frame_m=m, keep_k=k, rank_r=r)
        new = X[f][out["idx_f"]]
        n0 = kept_rows.shape[0]
        G = np.zeros((n0 + m, n0 + m))
        G[:n0, :n0] = G_keep
        G[n0:, :n0] = new @ kept_rows.T
        G[:n0, n0:] = G[n0:, :n0].T
        G[n0:, n0:] = new @ new.T
        if out["c"] is not None:
            lam, V = np.linalg.eigh(G)
            top = np.argsort(lam)[::-1][:r]
            Gr = (V[:, top] * lam[top]) @ V[:, top].T
            np.testing.assert_allclose(out["c"], np.diag(Gr), rtol=1e-9, atol=1e-12)
        G_keep = G[np.ix_(out["sel"], out["sel"])]
        np.testing.assert_allclose(G_keep, st.rows @ st.rows.T, rtol=1e-12, atol=1e-12)


def test_kept_set_invariants_over_many_frames():
    X, s = _frames(8, 40, 10, 3)
    st = S.empty_state(10)
    k, m, r = 25, 12, 4
    seen = {}
    n_keep = 0
    for f in range(8):
        out = S.stream_step(st, X[f], s[f], id_base=1000 * f, frame_m=m, keep_k=k, rank_r=r)
        for pos in out["idx_f"]:
            seen[1000 * f + int(pos)] = X[f][pos]
        n_keep = min(k, n_keep + m)
        assert st.ids.shape == (n_keep,) and st.rows.shape == (n_keep, 10)
        assert len(set(st.ids.tolist())) == n_keep                       # no token twice
        assert np.all(np.diff(out["sel"]) > 0)                           # candidate order is kept
        for i, row in zip(st.ids, st.rows):                              # rows travel with their ids, unchanged
            np.testing.assert_array_equal(row, seen[int(i)])
        if out["c"] is not None:
            dropped = np.setdiff1d(np.arange(out["c"].size), out["sel"])
            assert O.decision_values(out["c"])[out["sel"]].min() >= O.decision_values(out["c"])[dropped].max()


def test_a_token_outside_the_dominant_subspace_is_dropped_and_a_strong_one_survives():
    # candidates span two orthogonal directions with very different weight; with r = 1 only the heavy direction
    # carries energy, so tokens on the light direction are the first to go whatever frame they came from
    d = 6
    heavy, light = np.eye(d)[0], np.eye(d)[1]
    f0 = np.stack([3.0 * heavy, 2.5 * heavy, 0.2 * light, 2.0 * heavy])
    f1 = np.stack([0.1 * light, 2.8 * heavy, 0.3 * light])
    st = S.empty_state(d)
    S.stream_step(st, f0, np.array([0.9, 0.8, 0.7, 0.6]), id_base=0, frame_m=4, keep_k=4, rank_r=1)
    out = S.stream_step(st, f1, np.array([0.5, 0.9, 0.4]), id_base=10, frame_m=2, keep_k=4, rank_r=1)
    # candidates: ids 0, 1, 2, 3, then 10 and 11 (the two best-scored of the frame); energies 9, 6.25, 0, 4, 0, 7.84
    np.testing.assert_allclose(out["c"], [9.0, 6.25, 0.0, 4.0, 0.0, 7.84], atol=1e-12)
    np.testing.assert_array_equal(st.ids, [0, 1, 3, 11])
