"""covspec_verify_static (the entry point that allocates nothing: its scratch is a device array inside the
library) against covspec_verify on the same inputs, through the C ABI: two calls in a row, the second on a
smaller input, so that what the first call left in the shared array must not leak into the second."""
import numpy as np
import pytest

import covspec_inputs as I

pytestmark = pytest.mark.gpu


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)


def test_static_scratch_verify_matches_workspace_verify_on_two_calls():
    import torch
    import paper_2605_02218_amd as C
    C.load_library()
    # first call: several chunks per row and a ragged last one; second call: fewer, shorter rows
    for S, L, V, seed in ((24, 8, 3 * 8192 + 520, 11), (5, 3, 8192 + 264, 12)):
        p = C.VerifyParams(S, L, V, C.BF16)
        assert 0 < C.verify_workspace_size(p) <= C.VERIFY_STATIC_MAX_SCRATCH
        vb = I.make_verify_batch(S, L, V, I.BF16, seed=seed, copy_rows=1)
        zt, zd = _dev(vb["zt"]), _dev(vb["zd"])
        tok, ua, ur = (torch.from_numpy(vb[k]).cuda() for k in ("tok", "u_acc", "u_res"))
        n_ref, c_ref, a_ref = C.verify(p, zt, zd, tok, ua, ur)
        n_out = torch.full((S,), -7, dtype=torch.int32, device="cuda")
        c_out = torch.full((S,), -7, dtype=torch.int32, device="cuda")
        a_out = torch.full((S, L), -7.0, dtype=torch.float32, device="cuda")
        C.verify_static(p, zt, zd, tok, ua, ur, n_out, c_out, a_out)
        torch.cuda.synchronize()
        # integers bit-exact; alpha is the same arithmetic in the same order, hence bit-equal as well
        assert torch.equal(n_out, n_ref), "accepted counts differ (S=%d L=%d V=%d)" % (S, L, V)
        assert torch.equal(c_out, c_ref), "corrections differ (S=%d L=%d V=%d)" % (S, L, V)
        np.testing.assert_array_equal(a_out.cpu().numpy(), a_ref.cpu().numpy())
        assert (n_ref.cpu().numpy() < L).any() and (n_ref.cpu().numpy() > 0).any()   # the case exercises both outcomes


def test_static_scratch_verify_refuses_what_does_not_fit():
    import torch
    import paper_2605_02218_amd as C
    C.load_library()
    p = C.VerifyParams(4096, 15, 151936, C.BF16)         # 61440 rows: its partial sums exceed the array
    assert C.verify_workspace_size(p) > C.VERIFY_STATIC_MAX_SCRATCH
    one = torch.zeros(16, dtype=torch.int32, device="cuda")
    with pytest.raises(C.CovspecError) as err:
        C.verify_static(p, one, one, one, one, one, one, one, None)     # refused on the host: nothing is read
    assert err.value.status == C.binding.UNSUPPORTED
