"""Host-side checks of the C ABI: symbols, defaults, argument validation (no GPU work is launched)."""
import ctypes
import os
import re

import pytest

import paper_2605_02218_amd as C
from paper_2605_02218_amd import binding as Bd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "covspec.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(covspec_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = C.load_library()
    names = _declared_functions()
    assert set(names) == set(Bd.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_params_struct_layout_matches_header():
    assert ctypes.sizeof(Bd.CovspecParams) == 15 * 4


def _p(**kw):
    base = dict(batch=2, n_tokens=576, d_model=1024, n_query=16, n_heads=8, n_act_layers=4, dtype=C.FP32,
                keep_k=64, preselect_m=128, rank_r=32)
    base.update(kw)
    return C.Params(**base)


def test_resolve_defaults():
    assert C.resolve(_p()) == (64, 128, 32)
    assert C.resolve(_p(preselect_m=0, rank_r=0)) == (64, 128, 32)
    assert C.resolve(_p(n_tokens=8192, d_model=1536, keep_k=0, keep_ratio=0.1, preselect_m=0, rank_r=128)) == (819, 1638, 128)
    assert C.resolve(_p(keep_k=0, keep_ratio=1.0, preselect_m=0, rank_r=3)) == (576, 576, 3)
    assert C.workspace_size(_p()) > 0


@pytest.mark.parametrize("kw,status", [
    (dict(batch=0), Bd.INVALID_ARG), (dict(n_query=0), Bd.INVALID_ARG), (dict(n_heads=3), Bd.INVALID_ARG),
    (dict(dtype=2), Bd.INVALID_ARG), (dict(rel_mode=2), Bd.INVALID_ARG), (dict(lr_mode=-1), Bd.INVALID_ARG), (dict(lr_mode=4), Bd.INVALID_ARG),
    (dict(lam=1.5), Bd.INVALID_ARG), (dict(lam=float("nan")), Bd.INVALID_ARG),
    (dict(keep_k=200), Bd.INVALID_ARG),                       # k > M
    (dict(preselect_m=600), Bd.INVALID_ARG),                  # M > N
    (dict(rank_r=128), Bd.INVALID_ARG),                       # r >= min(M, d)
    (dict(keep_k=0, keep_ratio=0.0), Bd.INVALID_ARG),
    (dict(n_act_layers=-1), Bd.INVALID_ARG),
    (dict(n_tokens=20000), Bd.UNSUPPORTED), (dict(n_act_layers=9), Bd.UNSUPPORTED),
    (dict(d_model=1028, n_heads=1), Bd.OK), (dict(d_model=1026, n_heads=1), Bd.UNSUPPORTED),
    (dict(n_tokens=16384, keep_k=4097, preselect_m=8194, rank_r=8), Bd.UNSUPPORTED),
])
def test_invalid_params_are_rejected_on_the_host(kw, status):
    p = _p(**kw)
    cs = p.c_struct()
    lib = C.load_library()
    assert lib.covspec_resolve(ctypes.byref(cs), None, None, None) == status
    assert (C.workspace_size(p) > 0) == (status == Bd.OK)
    if status != Bd.OK:
        with pytest.raises(C.CovspecError):
            C.resolve(p)


def test_greedy_mode_does_not_need_a_rank():
    assert C.workspace_size(_p(lr_mode=C.LR_GREEDY_RESIDUAL, rank_r=128)) > 0


def test_ablation_selectors_need_no_rank_and_no_preselection_limit():
    assert C.workspace_size(_p(lr_mode=C.LR_SCORE_TOPK, rank_r=128)) > 0
    assert C.workspace_size(_p(lr_mode=C.LR_RANDOM, rank_r=128, seed=7)) > 0
    big = dict(n_tokens=16384, keep_k=4097, preselect_m=8194, rank_r=8)
    assert C.workspace_size(_p(lr_mode=C.LR_SCORE_TOPK, **big)) > 0
    assert C.workspace_size(_p(lr_mode=C.LR_SCORE_TOPK)) < C.workspace_size(_p())   # no low-rank buffers


def test_entry_points_reject_null_pointers_and_small_workspaces_before_any_launch():
    lib = C.load_library()
    p = _p()
    cs = p.c_struct()
    fake = 4096  # never dereferenced: validation fails first
    assert lib.covspec_score(ctypes.byref(cs), None, None, fake, None, None, None, None, None, fake, 1 << 40, None) == Bd.INVALID_ARG
    assert lib.covspec_select(ctypes.byref(cs), fake, fake, None, None, None, None, None, fake, 1 << 40, None) == Bd.INVALID_ARG
    assert lib.covspec_reduce(ctypes.byref(cs), fake, None, fake, None, None, fake, None, fake, 1 << 40, None) == Bd.INVALID_ARG
    assert lib.covspec_reduce(ctypes.byref(cs), fake, None, fake, None, None, fake, fake, fake, 16, None) == Bd.WORKSPACE_TOO_SMALL
    assert lib.covspec_reduce(ctypes.byref(cs), fake, None, fake, None, None, fake, fake, None, 1 << 40, None) == Bd.INVALID_ARG
    assert lib.covspec_reduce(ctypes.byref(cs), fake, None, fake, None, None, fake, fake, fake + 8, 1 << 40, None) == Bd.INVALID_ARG
    assert lib.covspec_score(None, fake, None, fake, None, None, None, None, None, fake, 1 << 40, None) == Bd.INVALID_ARG


def test_image_status_query_validates_on_the_host():
    lib = C.load_library()
    p = C.Params(batch=2, n_tokens=256, d_model=64, n_query=4, keep_k=16, preselect_m=32, rank_r=4)
    cs = p.c_struct()
    fake = 4096
    assert lib.covspec_image_status(ctypes.byref(cs), None, fake, None) == Bd.INVALID_ARG
    assert lib.covspec_image_status(ctypes.byref(cs), fake, None, None) == Bd.INVALID_ARG
    assert lib.covspec_image_status(ctypes.byref(cs), fake + 8, fake, None) == Bd.INVALID_ARG      # workspace alignment
    assert lib.covspec_image_status(None, fake, fake, None) == Bd.INVALID_ARG
    bad = C.Params(batch=2, n_tokens=256, d_model=64, n_query=4, keep_k=64, preselect_m=32).c_struct()
    assert lib.covspec_image_status(ctypes.byref(bad), fake, fake, None) == Bd.INVALID_ARG
    lib.covspec_set_wait_limit_us(5)      # host-side setting only; restored to the default right away
    lib.covspec_set_wait_limit_us(0)


def test_status_strings():
    assert C.status_string(0) == "ok"
    assert "workspace" in C.status_string(2)
    assert C.status_string(99) == "unknown status"


def test_verify_params_are_validated_on_the_host():
    lib = C.load_library()
    assert ctypes.sizeof(Bd.CovspecVerifyParams) == 4 * 4
    ok = C.VerifyParams(n_seq=4, n_draft=8, vocab=4096, dtype=C.BF16)
    assert C.verify_workspace_size(ok) > 0
    assert C.verify_workspace_size(C.VerifyParams(1, 1, 8, C.BF16)) > 0
    fake = 4096
    for bad, status in [(C.VerifyParams(0, 8, 4096), Bd.INVALID_ARG), (C.VerifyParams(4, 0, 4096), Bd.INVALID_ARG),
                        (C.VerifyParams(4, 8, 1), Bd.INVALID_ARG), (C.VerifyParams(4, 8, 4096, 3), Bd.INVALID_ARG),
                        (C.VerifyParams(4, 8, 4100, C.BF16), Bd.UNSUPPORTED), (C.VerifyParams(4, 8, 4098, C.FP32), Bd.UNSUPPORTED),
                        (C.VerifyParams(8192, 8, 4096), Bd.UNSUPPORTED), (C.VerifyParams(4, 65, 4096), Bd.UNSUPPORTED)]:
        assert C.verify_workspace_size(bad) == 0
        cs = bad.c_struct()
        assert lib.covspec_verify(ctypes.byref(cs), fake, fake, fake, fake, fake, fake, fake, None, fake, 1 << 40, None) == status
    assert C.verify_workspace_size(C.VerifyParams(4, 8, 4100, C.FP32)) > 0
    assert C.verify_workspace_size(C.VerifyParams(4, 8, 4096, C.FP16)) > 0 and C.verify_workspace_size(C.VerifyParams(4, 8, 4100, C.FP16)) == 0
    cs = ok.c_struct()
    assert lib.covspec_verify(ctypes.byref(cs), None, fake, fake, fake, fake, fake, fake, None, fake, 1 << 40, None) == Bd.INVALID_ARG
    assert lib.covspec_verify(ctypes.byref(cs), fake, fake, fake, fake, fake, None, fake, None, fake, 1 << 40, None) == Bd.INVALID_ARG
    assert lib.covspec_verify(ctypes.byref(cs), fake + 8, fake, fake, fake, fake, fake, fake, None, fake, 1 << 40, None) == Bd.INVALID_ARG
    assert lib.covspec_verify(ctypes.byref(cs), fake, fake, fake, fake, fake, fake, fake, None, fake, 16, None) == Bd.WORKSPACE_TOO_SMALL
    assert lib.covspec_verify(None, fake, fake, fake, fake, fake, fake, fake, None, fake, 1 << 40, None) == Bd.INVALID_ARG


def test_static_scratch_verify_validates_on_the_host():
    """covspec_verify_static refuses bad arguments and shapes beyond its array before it touches a device."""
    lib = C.load_library()
    fake = 4096
    big = C.VerifyParams(4096, 15, 151936, C.BF16)
    assert C.verify_workspace_size(big) > C.VERIFY_STATIC_MAX_SCRATCH
    cs = big.c_struct()
    assert lib.covspec_verify_static(ctypes.byref(cs), fake, fake, fake, fake, fake, fake, fake, None, None) == Bd.UNSUPPORTED
    assert b"static array" in lib.covspec_last_error()
    cs = C.VerifyParams(4, 8, 4096, C.BF16).c_struct()
    assert lib.covspec_verify_static(ctypes.byref(cs), None, fake, fake, fake, fake, fake, fake, None, None) == Bd.INVALID_ARG
    assert lib.covspec_verify_static(ctypes.byref(cs), fake, fake + 8, fake, fake, fake, fake, fake, None, None) == Bd.INVALID_ARG
    cs = C.VerifyParams(4, 65, 4096, C.BF16).c_struct()
    assert lib.covspec_verify_static(ctypes.byref(cs), fake, fake, fake, fake, fake, fake, fake, None, None) == Bd.UNSUPPORTED
    assert lib.covspec_verify_static(None, fake, fake, fake, fake, fake, fake, fake, None, None) == Bd.INVALID_ARG


def test_draft_params_validation_and_fanout_match_the_oracle_formula():
    """covspec_draft_fanout is host arithmetic: F_j = ceil(F_0 rho^j) must agree with the oracle's exact rational
    evaluation for every (F_0, rho) on a grid, exact powers of two and decimal rho whose products are exact
    integers included (rho is a double in the parameter block)."""
    from oracle import draft_oracle as DO
    assert ctypes.sizeof(Bd.CovspecDraftParams) == 40     # 5 int32, padding, double, float, padding
    for f0 in (0, 1, 2, 5, 8, 10, 16, 20, 30, 32):
        for rho in (0.5, 0.25, 0.6, 0.7, 0.9, 0.1, 0.2, 0.3, 0.05, 1 / 3, 0.999):
            p = C.DraftParams(n_seq=2, n_draft=12, vocab=4096, fanout0=f0, rho=rho)
            assert C.draft_fanout(p) == DO.fanout(f0, rho, 12), (f0, rho)
    assert C.draft_fanout(C.DraftParams(1, 3, 4096, fanout0=10, rho=0.1)) == [10, 1, 1]
    assert C.draft_fanout(C.DraftParams(1, 3, 4096, fanout0=30, rho=0.1)) == [30, 3, 1]
    assert C.draft_fanout(C.DraftParams(1, 6, 4096, fanout0=8, rho=0.5)) == [8, 4, 2, 1, 1, 1]
    lib = C.load_library()
    ok = C.DraftParams(4, 8, 8192)
    assert C.draft_workspace_size(ok) > 0
    fake = 4096
    for bad, status in [(C.DraftParams(0, 8, 8192), Bd.INVALID_ARG), (C.DraftParams(4, 8, 8192, rho=0.0), Bd.INVALID_ARG),
                        (C.DraftParams(4, 8, 8192, rho=1.5), Bd.INVALID_ARG), (C.DraftParams(4, 8, 8192, rho=1.0), Bd.INVALID_ARG), (C.DraftParams(4, 8, 8192, gamma=float("nan")), Bd.INVALID_ARG),
                        (C.DraftParams(4, 8, 8192, fanout0=-1), Bd.INVALID_ARG), (C.DraftParams(4, 8, 8192, fanout0=33), Bd.UNSUPPORTED),
                        (C.DraftParams(4, 65, 8192), Bd.UNSUPPORTED), (C.DraftParams(4, 8, 8196, C.BF16), Bd.UNSUPPORTED),
                        (C.DraftParams(4, 8, 524288 + 8), Bd.UNSUPPORTED), (C.DraftParams(2000, 64, 8192), Bd.UNSUPPORTED)]:
        assert C.draft_workspace_size(bad) == 0
        cs = bad.c_struct()
        assert lib.covspec_draft_gate(ctypes.byref(cs), fake, fake, fake, fake, fake, fake, 1 << 40, None) == status
    cs = ok.c_struct()
    assert lib.covspec_draft_gate(ctypes.byref(cs), None, fake, fake, fake, fake, fake, 1 << 40, None) == Bd.INVALID_ARG
    assert lib.covspec_draft_gate(ctypes.byref(cs), fake, fake, fake, fake, None, fake, 1 << 40, None) == Bd.INVALID_ARG
    assert lib.covspec_draft_gate(ctypes.byref(cs), fake, fake, fake, fake, fake, fake, 16, None) == Bd.WORKSPACE_TOO_SMALL
    assert lib.covspec_draft_gate(ctypes.byref(cs), fake + 4, fake, fake, fake, fake, fake, 1 << 40, None) == Bd.INVALID_ARG
    cs0 = C.DraftParams(4, 8, 8192, fanout0=0).c_struct()     # margin only: no candidate buffer needed
    assert lib.covspec_draft_gate(ctypes.byref(cs0), fake, fake, fake, fake, None, fake, 16, None) == Bd.WORKSPACE_TOO_SMALL


def test_ragged_resolution_runs_and_validation():
    p = _p(keep_k=0, preselect_m=0, rank_r=0, keep_ratio=0.25, d_model=256, n_heads=4)
    ks, runs = C.ragged_resolve(p, [256, 256, 512, 256, 768, 768, 768], [4, 4, 4, 9, 9, 9, 8])
    assert ks == [64, 64, 128, 64, 192, 192, 192] and runs == 5          # a run ends when N or T changes
    assert C.ragged_resolve(p, [300], [1]) == ([75], 1)
    for bad in ([256, 0], [256, 20000]):
        with pytest.raises(C.CovspecError):
            C.ragged_resolve(p, bad, [4, 4])
    with pytest.raises(ValueError):
        C.ragged_resolve(p, [256], [4, 4])
    lib = C.load_library()
    desc, keep = Bd._ragged_desc([256, 512], [4, 4])
    cs = p.c_struct()
    one = lib.covspec_ragged_workspace_size(ctypes.byref(cs), ctypes.byref(desc), 1)
    assert one > 0 and lib.covspec_ragged_workspace_size(ctypes.byref(cs), ctypes.byref(desc), 3) == 3 * one
    assert lib.covspec_ragged_workspace_size(ctypes.byref(cs), ctypes.byref(desc), 0) == 0
    fake = 4096
    streams = (ctypes.c_void_p * 1)(None)
    call = lambda *a: lib.covspec_reduce_ragged(ctypes.byref(cs), ctypes.byref(desc), *a)
    assert call(fake, None, fake, None, None, fake, fake, fake, 16, streams, 1) == Bd.WORKSPACE_TOO_SMALL
    assert call(None, None, fake, None, None, fake, fake, fake, 1 << 40, streams, 1) == Bd.INVALID_ARG
    assert call(fake, None, fake, None, None, fake, fake, fake, 1 << 40, None, 1) == Bd.INVALID_ARG
    assert call(fake, None, fake, None, None, fake, fake, fake, 1 << 40, streams, 0) == Bd.INVALID_ARG
    many = (ctypes.c_void_p * 9)(*([None] * 9))
    assert call(fake, None, fake, None, None, fake, fake, fake, 1 << 40, many, 9) == Bd.INVALID_ARG     # more than 8 streams


def test_stream_params_are_validated_on_the_host():
    assert ctypes.sizeof(Bd.CovspecStreamParams) == 7 * 4
    ok = dict(batch=2, n_frame=256, d_model=128, frame_m=64, keep_k=192, rank_r=16, dtype=C.BF16)
    assert C.stream_workspace_size(C.StreamParams(**ok)) > 0
    for bad in (dict(frame_m=0), dict(frame_m=257), dict(rank_r=0), dict(rank_r=128), dict(rank_r=192), dict(keep_k=0),
                dict(dtype=C.FP16), dict(batch=0), dict(d_model=100), dict(keep_k=4090), dict(n_frame=20000, frame_m=64)):
        assert C.stream_workspace_size(C.StreamParams(**{**ok, **bad})) == 0, bad
    lib = C.load_library()
    cs = C.StreamParams(**ok).c_struct()
    fake, big = 4096, 1 << 40
    call = lambda n_keep, *a: lib.covspec_stream_step(ctypes.byref(cs), n_keep, 0, *a)
    nxt = ctypes.c_int32(0)
    # n_keep outside 0..k; a missing required pointer; a missing input state with tokens kept; workspace too small / misaligned
    assert call(-1, fake, fake, fake, fake, fake, fake, fake, fake, None, ctypes.byref(nxt), fake, big, None) == Bd.INVALID_ARG
    assert call(193, fake, fake, fake, fake, fake, fake, fake, fake, None, ctypes.byref(nxt), fake, big, None) == Bd.INVALID_ARG
    assert call(0, None, fake, None, None, None, fake, fake, fake, None, ctypes.byref(nxt), fake, big, None) == Bd.INVALID_ARG
    assert call(5, fake, fake, None, fake, fake, fake, fake, fake, None, ctypes.byref(nxt), fake, big, None) == Bd.INVALID_ARG
    assert call(0, fake, fake, None, None, None, fake, fake, fake, None, ctypes.byref(nxt), fake, 16, None) == Bd.WORKSPACE_TOO_SMALL
    assert call(0, fake, fake, None, None, None, fake, fake, fake, None, ctypes.byref(nxt), fake + 8, big, None) == Bd.INVALID_ARG
