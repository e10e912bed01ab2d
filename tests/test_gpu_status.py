"""covspec_image_status: the per-image word that says whether the multi-workgroup kernels of the low-rank stage
ran to the end or gave up waiting for one another.  The give-up path is driven from the host by shortening the
wait limit to one microsecond: every kernel still exits normally (each wait is bounded and a failed wait only
ends the image's work early), nothing faults or hangs."""
import numpy as np
import pytest

import covspec_inputs as I
from tests import util as U

pytestmark = pytest.mark.gpu

W = I.small_workload(cid=17, name="status", batch=4, n_tokens=1300, d_model=256, dtype=I.BF16, n_query=6, n_heads=2,
                     keep_k=200, preselect_m=640, rank_r=64, factor_rank=200, n_act_layers=1)


@pytest.fixture(scope="module")
def C():
    import paper_2605_02218_amd as C
    C.load_library()
    return C


@pytest.mark.parametrize("lr_mode", [0, 1], ids=["energy", "greedy"])
def test_status_is_zero_after_a_normal_call_and_one_after_a_starved_wait(C, lr_mode):
    import torch
    batch = U.gen_batch(W)
    dev = U.upload(batch, W.dtype)
    p = U.lib_params(C, W, W.batch, rel_mode=0, lr_mode=lr_mode)
    ws = C.alloc_workspace(p)
    args = (p, dev["X"], dev["hidden"], dev["Q"], dev["Wq"], dev["Wk"])
    idx0, tok0 = C.reduce(*args, workspace=ws)
    st0 = C.image_status(p, ws)
    torch.cuda.synchronize()
    assert st0.cpu().numpy().tolist() == [0] * W.batch
    ref = U.oracle_image(W, batch, 0, U.oracle_params(W, rel_mode=0, lr_mode=lr_mode))
    np.testing.assert_array_equal(idx0[0].cpu().numpy(), ref["idx"])

    print("shortening the wait limit to 1 us (lr_mode %d)" % lr_mode, flush=True)
    C.set_wait_limit_us(1)
    try:
        idx1, tok1 = C.reduce(*args, workspace=ws)
        st1 = C.image_status(p, ws)
        torch.cuda.synchronize()
    finally:
        C.set_wait_limit_us(0)
    st1 = st1.cpu().numpy()
    idx1 = idx1.cpu().numpy()
    print("images that gave up:", st1.tolist(), flush=True)
    assert set(st1.tolist()) <= {0, 1}
    assert st1.sum() >= 1, "no image gave up although no workgroup waits longer than a microsecond"
    # whatever happened, the indices are valid positions (never out of range), ascending and unique
    assert idx1.min() >= 0 and idx1.max() < W.n_tokens and np.all(np.diff(idx1, axis=1) > 0)
    for b in range(W.batch):
        if st1[b] == 0:           # an image that did not give up has the normal result
            np.testing.assert_array_equal(idx1[b], idx0[b].cpu().numpy())

    # with the default limit restored the same workspace gives the normal result and a clear status again
    idx2, _ = C.reduce(*args, workspace=ws)
    st2 = C.image_status(p, ws)
    torch.cuda.synchronize()
    assert st2.cpu().numpy().tolist() == [0] * W.batch
    assert torch.equal(idx2, idx0)
