"""The entry points under HIP graph capture: nothing inside allocates, synchronises or records a memset node,
and the kernels that meet at global-memory barriers re-initialise their counters in every call, so a captured call
replays.  Each replay runs on new input contents and is checked against the oracle (and so against the eager call).
Between replays the test does eager work and synchronises, as a caller's loop would."""
import numpy as np
import pytest

import covspec_inputs as I
import util as U
from oracle import covspec_oracle as O

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("modes", [(0, 0), (1, 1)], ids=["paper", "variant"])
def test_reduce_replays_from_a_captured_graph(modes):
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_2605_02218_amd as C
    C.load_library()
    w = I.small_workload(cid=14, name="graph", batch=3, n_tokens=333, d_model=256, dtype=I.BF16, n_query=7, n_heads=2,
                         keep_k=24, preselect_m=56, rank_r=10, factor_rank=48, n_act_layers=4)
    over = dict(keep_k=min(w.keep_k, w.d_model // 2)) if modes[1] == 1 else {}
    p = U.lib_params(C, w, w.batch, rel_mode=modes[0], lr_mode=modes[1], **over)
    k, _, _ = C.resolve(p)
    wts = I.make_weights(w)
    Wq, Wk = U.to_device(wts["Wq"], w.dtype), U.to_device(wts["Wk"], w.dtype)
    # static buffers of the graph
    X = torch.empty(w.batch, w.n_tokens, w.d_model, dtype=torch.bfloat16, device="cuda")
    Hd = torch.empty(w.batch, w.n_act_layers + 1, w.n_tokens, w.d_model, dtype=torch.bfloat16, device="cuda")
    Q = torch.empty(w.batch, w.n_query, w.d_model, dtype=torch.bfloat16, device="cuda")
    idx = torch.empty(w.batch, k, dtype=torch.int32, device="cuda")
    tok = torch.empty(w.batch, k, w.d_model, dtype=torch.bfloat16, device="cuda")
    ws = C.alloc_workspace(p)

    def load(first_image):
        per = [I.make_image(w, first_image + b) for b in range(w.batch)]
        for name, dst in (("X", X), ("hidden", Hd), ("Q", Q)):
            dst.copy_(U.to_device(np.stack([q[name] for q in per]), w.dtype))
        return per

    per = load(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        C.reduce(p, X, Hd, Q, Wq, Wk, workspace=ws, idx_out=idx, tokens_out=tok)       # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        C.reduce(p, X, Hd, Q, Wq, Wk, workspace=ws, idx_out=idx, tokens_out=tok)
    op = U.oracle_params(w, rel_mode=modes[0], lr_mode=modes[1], **over)
    for replay in range(3):
        per = load(10 * replay)                      # eager copies into the graph's input buffers
        idx.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = idx.cpu().numpy()
        for b in range(w.batch):
            ref = O.reduce(I.as_f64(per[b]["X"], w.dtype), I.as_f64(per[b]["hidden"], w.dtype), I.as_f64(per[b]["Q"], w.dtype),
                           I.as_f64(wts["Wq"], w.dtype), I.as_f64(wts["Wk"], w.dtype), op)
            np.testing.assert_array_equal(got[b], ref["idx"], err_msg="replay %d image %d" % (replay, b))
            rows = tok[b].view(torch.int16).cpu().numpy().view(np.uint16)
            np.testing.assert_array_equal(rows, per[b]["X"][got[b]])
