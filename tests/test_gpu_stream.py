"""Parity of covspec_stream_step (frame-by-frame selection with a carried Gram matrix) against oracle/stream_oracle.py."""
import numpy as np
import pytest

import covspec_inputs as I
from oracle import stream_oracle as S

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def C():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_2605_02218_amd as C
    C.load_library()
    return C


def _dev(a, dtype):
    import torch
    if dtype == I.BF16:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def _run(C, B, n_frames, n_frame, d, m, k, r, dtype, cut_every=0, factor_rank=64, seed0=None):
    """Drives B videos through n_frames frames on the GPU and in the oracle; checks every frame."""
    import torch
    seed0 = 10 * B if seed0 is None else seed0
    vids = [I.make_video_stream(n_frames, n_frame, d, dtype=dtype, seed=seed0 + b, cut_every=cut_every,
                                factor_rank=factor_rank) for b in range(B)]
    p = C.StreamParams(batch=B, n_frame=n_frame, d_model=d, frame_m=m, keep_k=k, rank_r=r, dtype=dtype)
    ws = torch.empty(C.stream_workspace_size(p) + 256, dtype=torch.uint8, device="cuda")
    states = [C.stream_alloc_state(p), C.stream_alloc_state(p)]
    ora = [S.empty_state(d) for _ in range(B)]
    n_keep, solved = 0, 0
    tol = 1e-5      # of the largest energy: the rows are given exactly, the Gram matrix and the solve are fp64-grade
    for f in range(n_frames):
        Xf = np.stack([v[0][f] for v in vids])
        sf = np.stack([v[1][f] for v in vids])
        src, dst = states[f & 1], states[(f + 1) & 1]
        nxt, c = C.stream_step(p, n_keep, f * n_frame, _dev(Xf, dtype), torch.from_numpy(sf).cuda(),
                               src if n_keep else None, dst, workspace=ws, want_c=True)
        torch.cuda.synchronize()
        assert nxt == min(k, n_keep + m)
        Z, G, ids = (t.cpu() for t in dst)
        for b in range(B):
            ref = S.stream_step(ora[b], I.as_f64(Xf[b], dtype), sf[b], f * n_frame, m, k, r)
            where = "frame %d video %d" % (f, b)
            if ref["c"] is not None:
                solved += 1
                assert ref["margin_topk"] > 2e-5 and ref["sigma_gap"] > 1e-4, "%s: input has a near-tie: %r" % (where, ref)
                got = c[b].cpu().numpy().astype(np.float64)
                scale = max(np.abs(ref["c"]).max(), 1e-300)
                np.testing.assert_allclose(got / scale, ref["c"] / scale, atol=tol, rtol=0, err_msg=where)
            else:
                assert c is None
            np.testing.assert_array_equal(ids[b, :nxt].numpy(), ref["ids"], err_msg=where)
            rows = Z[b, :nxt].view(torch.int16).numpy() if dtype == I.BF16 else Z[b, :nxt].numpy()
            want = I.store(ora[b].rows.astype(np.float32), dtype)
            np.testing.assert_array_equal(rows, want.view(np.int16) if dtype == I.BF16 else want, err_msg=where)
            # the carried Gram matrix is that of the kept rows: bf16 products are exact and summed in fp32 pieces
            # flushed into fp64 (relative 1e-6 of the row norms); fp32 storage is contracted in fp64
            Gref = ora[b].rows @ ora[b].rows.T
            gs = np.sqrt(np.outer(np.diag(Gref), np.diag(Gref)))
            np.testing.assert_allclose(G[b, :nxt, :nxt].numpy() / gs, Gref / gs, atol=2e-6 if dtype == I.BF16 else 1e-12,
                                       rtol=0, err_msg=where)
        n_keep = nxt
    return solved


def test_stream_matches_oracle_bf16_subspace_iteration(C):
    # k + M_f = 320 candidates, r = 24: block iteration (block of 128); 7 frames: 2 of warm-up, 5 with a decision
    assert _run(C, B=3, n_frames=7, n_frame=200, d=256, m=96, k=224, r=24, dtype=I.BF16) == 15


def test_stream_matches_oracle_fp32_full_solve_and_scene_cuts(C):
    # 150 candidates, r = 60: the full Jacobi solve; a fresh scene every third frame; M_f does not divide k, so the
    # first decision sees fewer candidates than the later ones
    assert _run(C, B=2, n_frames=8, n_frame=130, d=96, m=50, k=100, r=30, dtype=I.FP32, cut_every=3) >= 10


def test_stream_keeps_everything_while_the_memory_is_not_full(C):
    # k is never reached: every frame only appends (no eigen-solve), ids and rows in arrival order
    assert _run(C, B=2, n_frames=3, n_frame=64, d=64, m=16, k=64, r=4, dtype=I.BF16) == 0


def test_stream_frame_m_equals_n_frame_and_single_video(C):
    # no pre-selection inside the frame (M_f = N_f), one video
    assert _run(C, B=1, n_frames=4, n_frame=72, d=128, m=72, k=100, r=10, dtype=I.FP32) == 3


def test_stream_at_the_benchmark_shape(C):
    # the shape bench.py --stream times: 4 videos, frames of 1024 x 1536 bf16, 256 pre-selected, 1024 kept, r = 128;
    # four frames fill the memory, two decide among 1280 candidates (block iteration with a block of 192)
    # (the videos of the benchmark: seeds 0..3)
    assert _run(C, B=4, n_frames=6, n_frame=1024, d=1536, m=256, k=1024, r=128, dtype=I.BF16, seed0=0) == 8
