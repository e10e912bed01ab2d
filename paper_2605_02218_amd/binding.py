"""ctypes binding of libcovspec.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI declared in
include/covspec.h; this module converts torch tensors to device pointers,
supplies the current HIP stream and allocates outputs / workspace.  There is
no CPU fallback: a missing library raises at import of the symbols.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libcovspec.so")

FP32, BF16 = 0, 1
FP16 = 2          # logits of verify / draft_gate only
REL_COSINE_MAX, REL_ATTN_SOFTMAX = 0, 1
LR_ENERGY_TOPK, LR_GREEDY_RESIDUAL, LR_SCORE_TOPK, LR_RANDOM = 0, 1, 2, 3
OK, INVALID_ARG, WORKSPACE_TOO_SMALL, UNSUPPORTED, HIP_ERROR = 0, 1, 2, 3, 4

EXPORTS = ("covspec_workspace_size", "covspec_resolve", "covspec_score", "covspec_select",
           "covspec_reduce", "covspec_reduce_staged", "covspec_probe_launches", "covspec_status_string",
           "covspec_verify_workspace_size", "covspec_verify", "covspec_verify_static", "covspec_draft_fanout", "covspec_draft_workspace_size",
           "covspec_draft_gate", "covspec_last_error", "covspec_ragged_resolve", "covspec_ragged_workspace_size",
           "covspec_reduce_ragged", "covspec_lowrank_path", "covspec_image_status", "covspec_set_wait_limit_us", "covspec_stream_workspace_size", "covspec_stream_step")


class CovspecParams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "batch", "n_tokens", "d_model", "n_query", "n_heads", "n_act_layers", "dtype",
        "rel_mode", "lr_mode", "preselect_m", "rank_r", "keep_k")] + [
        ("keep_ratio", ctypes.c_float), ("lambda_", ctypes.c_float), ("seed", ctypes.c_uint32)]


class CovspecVerifyParams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("n_seq", "n_draft", "vocab", "dtype")]


class CovspecDraftParams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("n_seq", "n_draft", "vocab", "dtype", "fanout0")] + [
        ("rho", ctypes.c_double), ("gamma", ctypes.c_float)]


class CovspecRagged(ctypes.Structure):
    _fields_ = [("n_images", ctypes.c_int32), ("n_tokens", ctypes.POINTER(ctypes.c_int32)),
                ("n_query", ctypes.POINTER(ctypes.c_int32))]


class CovspecStreamParams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("batch", "n_frame", "d_model", "dtype", "frame_m", "keep_k", "rank_r")]


class CovspecError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = load_library().covspec_last_error().decode() if status == HIP_ERROR else ""
        super().__init__("%s: %s (status %d)%s" % (where, status_string(status), status, " [" + detail + "]" if detail else ""))


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libcovspec.so (built by paper_2605_02218_amd.build); fail loudly if absent."""
    global _lib
    if _lib is not None:
        return _lib
    # PyTorch ships its own copy of the HIP runtime.  It has to be in the process BEFORE this library is opened,
    # so that both bind to the same runtime: opened first, the library would pull in the system's copy, and its
    # launches would then run against a runtime that knows nothing of torch's device memory and streams
    # (every launch fails with hipErrorNoDevice).
    import torch  # noqa: F401
    if not os.path.exists(LIB_PATH):
        raise ImportError("%s not found: run `python -m paper_2605_02218_amd.build` (or __graft_entry__.build()) first"
                          % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, pp = ctypes.c_void_p, ctypes.POINTER(CovspecParams)
    lib.covspec_workspace_size.restype = ctypes.c_size_t
    lib.covspec_workspace_size.argtypes = [pp]
    lib.covspec_resolve.restype = ctypes.c_int
    lib.covspec_resolve.argtypes = [pp] + [ctypes.POINTER(ctypes.c_int32)] * 3
    lib.covspec_score.restype = ctypes.c_int
    lib.covspec_score.argtypes = [pp] + [vp] * 8 + [vp, ctypes.c_size_t, vp]
    lib.covspec_select.restype = ctypes.c_int
    lib.covspec_select.argtypes = [pp] + [vp] * 7 + [vp, ctypes.c_size_t, vp]
    lib.covspec_reduce.restype = ctypes.c_int
    lib.covspec_reduce.argtypes = [pp] + [vp] * 7 + [vp, ctypes.c_size_t, vp]
    lib.covspec_reduce_staged.restype = ctypes.c_int
    lib.covspec_reduce_staged.argtypes = [pp] + [vp] * 7 + [vp, ctypes.c_size_t, vp, ctypes.POINTER(vp)]
    lib.covspec_probe_launches.restype = ctypes.c_int
    lib.covspec_probe_launches.argtypes = [pp] + [ctypes.POINTER(ctypes.c_int32)] * 3
    vpp = ctypes.POINTER(CovspecVerifyParams)
    lib.covspec_verify_workspace_size.restype = ctypes.c_size_t
    lib.covspec_verify_workspace_size.argtypes = [vpp]
    lib.covspec_verify.restype = ctypes.c_int
    lib.covspec_verify.argtypes = [vpp] + [vp] * 8 + [vp, ctypes.c_size_t, vp]
    lib.covspec_verify_static.restype = ctypes.c_int
    lib.covspec_verify_static.argtypes = [vpp] + [vp] * 8 + [vp]
    dpp = ctypes.POINTER(CovspecDraftParams)
    lib.covspec_draft_fanout.restype = ctypes.c_int
    lib.covspec_draft_fanout.argtypes = [dpp, ctypes.POINTER(ctypes.c_int32)]
    lib.covspec_draft_workspace_size.restype = ctypes.c_size_t
    lib.covspec_draft_workspace_size.argtypes = [dpp]
    lib.covspec_draft_gate.restype = ctypes.c_int
    lib.covspec_draft_gate.argtypes = [dpp] + [vp] * 5 + [vp, ctypes.c_size_t, vp]
    lib.covspec_status_string.restype = ctypes.c_char_p
    lib.covspec_status_string.argtypes = [ctypes.c_int]
    rp = ctypes.POINTER(CovspecRagged)
    lib.covspec_ragged_resolve.restype = ctypes.c_int
    lib.covspec_ragged_resolve.argtypes = [pp, rp, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
    lib.covspec_ragged_workspace_size.restype = ctypes.c_size_t
    lib.covspec_ragged_workspace_size.argtypes = [pp, rp, ctypes.c_int32]
    lib.covspec_reduce_ragged.restype = ctypes.c_int
    lib.covspec_reduce_ragged.argtypes = [pp, rp] + [vp] * 7 + [vp, ctypes.c_size_t, ctypes.POINTER(vp), ctypes.c_int32]
    lib.covspec_lowrank_path.restype = ctypes.c_int
    lib.covspec_lowrank_path.argtypes = [pp, vp, vp, vp]
    lib.covspec_image_status.restype = ctypes.c_int
    lib.covspec_image_status.argtypes = [pp, vp, vp, vp]
    lib.covspec_set_wait_limit_us.restype = None
    lib.covspec_set_wait_limit_us.argtypes = [ctypes.c_int64]
    spp = ctypes.POINTER(CovspecStreamParams)
    lib.covspec_stream_workspace_size.restype = ctypes.c_size_t
    lib.covspec_stream_workspace_size.argtypes = [spp]
    lib.covspec_stream_step.restype = ctypes.c_int
    lib.covspec_stream_step.argtypes = [spp, ctypes.c_int32, ctypes.c_int32] + [vp] * 9 + [ctypes.POINTER(ctypes.c_int32), vp, ctypes.c_size_t, vp]
    lib.covspec_last_error.restype = ctypes.c_char_p
    lib.covspec_last_error.argtypes = []
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().covspec_status_string(int(status)).decode()


@dataclass
class Params:
    batch: int
    n_tokens: int
    d_model: int
    n_query: int
    n_heads: int = 1
    n_act_layers: int = 0
    dtype: int = BF16
    rel_mode: int = REL_COSINE_MAX
    lr_mode: int = LR_ENERGY_TOPK
    preselect_m: int = 0
    rank_r: int = 0
    keep_k: int = 0
    keep_ratio: float = 0.25
    lam: float = 0.5
    seed: int = 0

    def c_struct(self) -> CovspecParams:
        return CovspecParams(self.batch, self.n_tokens, self.d_model, self.n_query, self.n_heads,
                             self.n_act_layers, self.dtype, self.rel_mode, self.lr_mode, self.preselect_m,
                             self.rank_r, self.keep_k, self.keep_ratio, self.lam, self.seed & 0xFFFFFFFF)


def workspace_size(p: Params) -> int:
    cs = p.c_struct()
    return int(load_library().covspec_workspace_size(ctypes.byref(cs)))


def resolve(p: Params):
    """(k, M, r) after the library's defaults; raises CovspecError on invalid params."""
    cs = p.c_struct()
    k, m, r = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    st = load_library().covspec_resolve(ctypes.byref(cs), ctypes.byref(k), ctypes.byref(m), ctypes.byref(r))
    if st != OK:
        raise CovspecError(st, "covspec_resolve")
    return k.value, m.value, r.value


# ---------------------------------------------------------------- torch-facing helpers
def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous device tensors")
    return t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _torch_dtype(dtype: int):
    import torch
    return torch.bfloat16 if dtype == BF16 else torch.float32


def alloc_workspace(p: Params, device="cuda"):
    import torch
    n = workspace_size(p)
    if n == 0:
        cs = p.c_struct()
        st = load_library().covspec_resolve(ctypes.byref(cs), None, None, None)
        raise CovspecError(st if st != OK else INVALID_ARG, "covspec_workspace_size")
    return torch.empty(n + 256, dtype=torch.uint8, device=device)


def _ws_args(ws):
    base = ws.data_ptr()
    aligned = (base + 255) // 256 * 256
    return aligned, ws.numel() - (aligned - base)


def score(p: Params, X, hidden, Q, Wq, Wk, workspace=None):
    """covspec_score: returns (s_query, s_act or None, s_fused), each [B, N] fp32."""
    import torch
    ws = workspace if workspace is not None else alloc_workspace(p, X.device)
    B, N = p.batch, p.n_tokens
    sq = torch.empty(B, N, dtype=torch.float32, device=X.device)
    sf = torch.empty_like(sq)
    has_act = hidden is not None and p.n_act_layers > 0
    sa = torch.empty_like(sq) if has_act else None
    wp, wb = _ws_args(ws)
    cs = p.c_struct()
    st = load_library().covspec_score(ctypes.byref(cs), _ptr(X), _ptr(hidden), _ptr(Q), _ptr(Wq), _ptr(Wk),
                                      _ptr(sq), _ptr(sa), _ptr(sf), wp, wb, _stream())
    if st != OK:
        raise CovspecError(st, "covspec_score")
    return sq, sa, sf


def select(p: Params, X, s_fused, workspace=None):
    """covspec_select: dict with idx [B,k], idx_m [B,M] and c [B,M] (energy) or pick_order/resid [B,k] (greedy)."""
    import torch
    ws = workspace if workspace is not None else alloc_workspace(p, X.device)
    k, M, _ = resolve(p)
    B = p.batch
    dev = X.device
    idx = torch.empty(B, k, dtype=torch.int32, device=dev)
    idx_m = torch.empty(B, M, dtype=torch.int32, device=dev)
    out = {"idx": idx, "idx_m": idx_m}
    c = pick = resid = None
    if p.lr_mode == LR_ENERGY_TOPK:
        c = torch.empty(B, M, dtype=torch.float32, device=dev)
        out["c"] = c
    elif p.lr_mode == LR_RANDOM:
        idx_m = None
        del out["idx_m"]
    elif p.lr_mode == LR_SCORE_TOPK:
        pass
    else:
        pick = torch.empty(B, k, dtype=torch.int32, device=dev)
        resid = torch.empty(B, k, dtype=torch.float32, device=dev)
        out["pick_order"], out["resid"] = pick, resid
    wp, wb = _ws_args(ws)
    cs = p.c_struct()
    st = load_library().covspec_select(ctypes.byref(cs), _ptr(X), _ptr(s_fused), _ptr(idx), _ptr(c), _ptr(idx_m),
                                       _ptr(pick), _ptr(resid), wp, wb, _stream())
    if st != OK:
        raise CovspecError(st, "covspec_select")
    return out


STAGES = ("query_side", "token_projection", "relevance", "activity", "fuse", "preselect", "gram", "lowrank",
          "keep", "gather")
PROBE_BEGIN = len(STAGES) + 1       # event indices of the probed launch
PROBE_END = len(STAGES) + 2
NUM_STAGE_EVENTS = len(STAGES) + 3


def probe_launches(p: Params):
    """covspec_probe_launches: (equal launches per call, rows, cols, inner) of the probed fp64 product."""
    cs = p.c_struct()
    r, c, k = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int32(0)
    n = load_library().covspec_probe_launches(ctypes.byref(cs), ctypes.byref(r), ctypes.byref(c), ctypes.byref(k))
    return n, r.value, c.value, k.value


def reduce(p: Params, X, hidden, Q, Wq, Wk, workspace=None, idx_out=None, tokens_out=None, stage_events=None):
    """covspec_reduce: returns (idx [B,k] int32, tokens [B,k,d] in X's dtype).

    With `stage_events` (NUM_STAGE_EVENTS torch.cuda.Event objects, timing enabled, each recorded at least
    once before so that its handle exists) covspec_reduce_staged is called and the events mark the stages.
    """
    import torch
    ws = workspace if workspace is not None else alloc_workspace(p, X.device)
    k, _, _ = resolve(p)
    idx = idx_out if idx_out is not None else torch.empty(p.batch, k, dtype=torch.int32, device=X.device)
    tok = tokens_out if tokens_out is not None else torch.empty(p.batch, k, p.d_model, dtype=X.dtype, device=X.device)
    wp, wb = _ws_args(ws)
    cs = p.c_struct()
    if stage_events is None:
        st = load_library().covspec_reduce(ctypes.byref(cs), _ptr(X), _ptr(hidden), _ptr(Q), _ptr(Wq), _ptr(Wk),
                                           _ptr(idx), _ptr(tok), wp, wb, _stream())
    else:
        if len(stage_events) != NUM_STAGE_EVENTS:
            raise ValueError("need %d stage events" % NUM_STAGE_EVENTS)
        handles = (ctypes.c_void_p * NUM_STAGE_EVENTS)(*[e.cuda_event for e in stage_events])
        st = load_library().covspec_reduce_staged(ctypes.byref(cs), _ptr(X), _ptr(hidden), _ptr(Q), _ptr(Wq),
                                                  _ptr(Wk), _ptr(idx), _ptr(tok), wp, wb, _stream(), handles)
    if st != OK:
        raise CovspecError(st, "covspec_reduce")
    return idx, tok


@dataclass
class VerifyParams:
    n_seq: int
    n_draft: int
    vocab: int
    dtype: int = BF16

    def c_struct(self) -> CovspecVerifyParams:
        return CovspecVerifyParams(self.n_seq, self.n_draft, self.vocab, self.dtype)


def verify_workspace_size(p: VerifyParams) -> int:
    cs = p.c_struct()
    return int(load_library().covspec_verify_workspace_size(ctypes.byref(cs)))


def verify(p: VerifyParams, z_target, z_draft, tokens, u_accept, u_resample, workspace=None, want_alpha=True):
    """covspec_verify: returns (n_accept [S] int32, correction [S] int32, alpha [S, L] fp32 or None)."""
    import torch
    dev = z_target.device
    if workspace is None:
        n = verify_workspace_size(p)
        if n == 0:
            raise CovspecError(INVALID_ARG, "covspec_verify_workspace_size")
        workspace = torch.empty(n + 256, dtype=torch.uint8, device=dev)
    n_acc = torch.empty(p.n_seq, dtype=torch.int32, device=dev)
    corr = torch.empty(p.n_seq, dtype=torch.int32, device=dev)
    alpha = torch.empty(p.n_seq, p.n_draft, dtype=torch.float32, device=dev) if want_alpha else None
    wp, wb = _ws_args(workspace)
    cs = p.c_struct()
    st = load_library().covspec_verify(ctypes.byref(cs), _ptr(z_target), _ptr(z_draft), _ptr(tokens), _ptr(u_accept),
                                       _ptr(u_resample), _ptr(n_acc), _ptr(corr), _ptr(alpha), wp, wb, _stream())
    if st != OK:
        raise CovspecError(st, "covspec_verify")
    return n_acc, corr, alpha


VERIFY_STATIC_MAX_SCRATCH = 1 << 20


def verify_static(p: VerifyParams, z_target, z_draft, tokens, u_accept, u_resample, n_accept_out, correction_out,
                  alpha_out=None):
    """covspec_verify_static: as verify(), with the scratch in the library's own device array and every output
    supplied by the caller, so that the call allocates nothing."""
    cs = p.c_struct()
    st = load_library().covspec_verify_static(ctypes.byref(cs), _ptr(z_target), _ptr(z_draft), _ptr(tokens),
                                              _ptr(u_accept), _ptr(u_resample), _ptr(n_accept_out),
                                              _ptr(correction_out), _ptr(alpha_out), _stream())
    if st != OK:
        raise CovspecError(st, "covspec_verify_static")
    return n_accept_out, correction_out, alpha_out


@dataclass
class DraftParams:
    n_seq: int
    n_draft: int
    vocab: int
    dtype: int = BF16
    fanout0: int = 8
    rho: float = 0.5
    gamma: float = 0.5

    def c_struct(self) -> CovspecDraftParams:
        return CovspecDraftParams(self.n_seq, self.n_draft, self.vocab, self.dtype, self.fanout0, self.rho, self.gamma)


def draft_fanout(p: DraftParams):
    """covspec_draft_fanout: [F_0, ..., F_{L-1}]."""
    cs = p.c_struct()
    out = (ctypes.c_int32 * max(p.n_draft, 1))()
    st = load_library().covspec_draft_fanout(ctypes.byref(cs), out)
    if st != OK:
        raise CovspecError(st, "covspec_draft_fanout")
    return list(out)[:p.n_draft]


def draft_workspace_size(p: DraftParams) -> int:
    cs = p.c_struct()
    return int(load_library().covspec_draft_workspace_size(ctypes.byref(cs)))


def draft_gate(p: DraftParams, z_draft, tokens, workspace=None):
    """covspec_draft_gate: returns (margin [S, L] fp32, gate [S, L] int32, cand [S, L, F0] int32 or None)."""
    import torch
    dev = z_draft.device
    if workspace is None:
        n = draft_workspace_size(p)
        if n == 0:
            raise CovspecError(INVALID_ARG, "covspec_draft_workspace_size")
        workspace = torch.empty(n + 256, dtype=torch.uint8, device=dev)
    margin = torch.empty(p.n_seq, p.n_draft, dtype=torch.float32, device=dev)
    gate = torch.empty(p.n_seq, p.n_draft, dtype=torch.int32, device=dev)
    cand = torch.empty(p.n_seq, p.n_draft, p.fanout0, dtype=torch.int32, device=dev) if p.fanout0 > 0 else None
    wp, wb = _ws_args(workspace)
    cs = p.c_struct()
    st = load_library().covspec_draft_gate(ctypes.byref(cs), _ptr(z_draft), _ptr(tokens), _ptr(margin), _ptr(gate), _ptr(cand),
                                           wp, wb, _stream())
    if st != OK:
        raise CovspecError(st, "covspec_draft_gate")
    return margin, gate, cand


def _ragged_desc(n_tokens, n_query):
    n = len(n_tokens)
    if n != len(n_query):
        raise ValueError("n_tokens and n_query must have one entry per image")
    nt = (ctypes.c_int32 * max(n, 1))(*[int(v) for v in n_tokens])
    nq = (ctypes.c_int32 * max(n, 1))(*[int(v) for v in n_query])
    desc = CovspecRagged(n, ctypes.cast(nt, ctypes.POINTER(ctypes.c_int32)), ctypes.cast(nq, ctypes.POINTER(ctypes.c_int32)))
    return desc, (nt, nq)          # the arrays must outlive the descriptor


def ragged_resolve(p: Params, n_tokens, n_query):
    """covspec_ragged_resolve: (k per image, number of runs)."""
    desc, keep = _ragged_desc(n_tokens, n_query)
    cs = p.c_struct()
    ks = (ctypes.c_int32 * max(desc.n_images, 1))()
    runs = ctypes.c_int32(0)
    st = load_library().covspec_ragged_resolve(ctypes.byref(cs), ctypes.byref(desc), ks, ctypes.byref(runs))
    if st != OK:
        raise CovspecError(st, "covspec_ragged_resolve")
    return list(ks)[:desc.n_images], runs.value


def ragged_workspace_size(p: Params, n_tokens, n_query, n_streams: int = 1) -> int:
    desc, keep = _ragged_desc(n_tokens, n_query)
    cs = p.c_struct()
    return int(load_library().covspec_ragged_workspace_size(ctypes.byref(cs), ctypes.byref(desc), n_streams))


def reduce_ragged(p: Params, n_tokens, n_query, X, hidden, Q, Wq, Wk, streams=None, workspace=None, idx_out=None,
                  tokens_out=None, sync=True):
    """covspec_reduce_ragged on packed tensors: returns (idx [sum k_b] int32, tokens [sum k_b, d], k per image).

    `streams`: torch.cuda.Stream objects the runs are dealt to (default: the current stream only).  With several
    streams the inputs must be visible to all of them; they are synchronised before returning unless
    `sync=False` (then the caller owns `workspace` and synchronises)."""
    import torch
    ks, _ = ragged_resolve(p, n_tokens, n_query)
    desc, keep = _ragged_desc(n_tokens, n_query)
    cs = p.c_struct()
    handles = [s.cuda_stream for s in streams] if streams else [_stream()]
    ns = len(handles)
    if workspace is None:
        if streams and not sync:
            raise ValueError("sync=False with several streams needs a caller-owned workspace")
        need = int(load_library().covspec_ragged_workspace_size(ctypes.byref(cs), ctypes.byref(desc), ns))
        workspace = torch.empty(need + 256, dtype=torch.uint8, device=X.device)
    total = sum(ks)
    idx = idx_out if idx_out is not None else torch.empty(total, dtype=torch.int32, device=X.device)
    tok = tokens_out if tokens_out is not None else torch.empty(total, p.d_model, dtype=X.dtype, device=X.device)
    wp, wb = _ws_args(workspace)
    harr = (ctypes.c_void_p * ns)(*handles)
    st = load_library().covspec_reduce_ragged(ctypes.byref(cs), ctypes.byref(desc), _ptr(X), _ptr(hidden), _ptr(Q), _ptr(Wq),
                                              _ptr(Wk), _ptr(idx), _ptr(tok), wp, wb, harr, ns)
    if st != OK:
        raise CovspecError(st, "covspec_reduce_ragged")
    if streams and sync:
        for s in streams:
            s.synchronize()
    return idx, tok, ks


def lowrank_path(p: Params, workspace):
    """covspec_lowrank_path: int32 [B] tensor, the eigen-solve path of each image in the last call on `workspace`."""
    import torch
    out = torch.empty(p.batch, dtype=torch.int32, device=workspace.device)
    wp, _ = _ws_args(workspace)
    cs = p.c_struct()
    st = load_library().covspec_lowrank_path(ctypes.byref(cs), wp, _ptr(out), _stream())
    if st != OK:
        raise CovspecError(st, "covspec_lowrank_path")
    return out


def image_status(p: Params, workspace):
    """covspec_image_status: int32 [B] tensor, 0 = valid, 1 = the image's multi-workgroup kernels gave up waiting."""
    import torch
    out = torch.empty(p.batch, dtype=torch.int32, device=workspace.device)
    wp, _ = _ws_args(workspace)
    cs = p.c_struct()
    st = load_library().covspec_image_status(ctypes.byref(cs), wp, _ptr(out), _stream())
    if st != OK:
        raise CovspecError(st, "covspec_image_status")
    return out


def set_wait_limit_us(microseconds: int) -> None:
    """covspec_set_wait_limit_us: wait limit of the multi-workgroup kernels (<= 0 restores the default)."""
    load_library().covspec_set_wait_limit_us(int(microseconds))


@dataclass
class StreamParams:
    batch: int
    n_frame: int
    d_model: int
    frame_m: int
    keep_k: int
    rank_r: int
    dtype: int = BF16

    def c_struct(self) -> CovspecStreamParams:
        return CovspecStreamParams(self.batch, self.n_frame, self.d_model, self.dtype, self.frame_m, self.keep_k, self.rank_r)


def stream_workspace_size(p: StreamParams) -> int:
    cs = p.c_struct()
    return int(load_library().covspec_stream_workspace_size(ctypes.byref(cs)))


def stream_alloc_state(p: StreamParams, device="cuda"):
    """One set of state buffers (Z [B,k,d], G [B,k,k] fp64, ids [B,k] int32); a caller keeps two and swaps them."""
    import torch
    return (torch.empty(p.batch, p.keep_k, p.d_model, dtype=_torch_dtype(p.dtype), device=device),
            torch.empty(p.batch, p.keep_k, p.keep_k, dtype=torch.float64, device=device),
            torch.empty(p.batch, p.keep_k, dtype=torch.int32, device=device))


def stream_step(p: StreamParams, n_keep: int, id_base: int, X_frame, s_fused, state_in, state_out, workspace=None, want_c=False):
    """covspec_stream_step: advances every video by one frame.  state_in / state_out are (Z, G, ids) tuples that
    must not share memory (state_in may be None while n_keep == 0).  Returns (n_keep_next, c or None)."""
    import torch
    if workspace is None:
        n = stream_workspace_size(p)
        if n == 0:
            raise CovspecError(INVALID_ARG, "covspec_stream_workspace_size")
        workspace = torch.empty(n + 256, dtype=torch.uint8, device=X_frame.device)
    wp, wb = _ws_args(workspace)
    zi, gi, ii = state_in if state_in is not None else (None, None, None)
    zo, go, io = state_out
    c = torch.empty(p.batch, n_keep + p.frame_m, dtype=torch.float32, device=X_frame.device) if want_c else None
    nxt = ctypes.c_int32(-1)
    cs = p.c_struct()
    st = load_library().covspec_stream_step(ctypes.byref(cs), n_keep, id_base, _ptr(X_frame), _ptr(s_fused), _ptr(zi), _ptr(gi),
                                            _ptr(ii), _ptr(zo), _ptr(go), _ptr(io), _ptr(c), ctypes.byref(nxt), wp, wb, _stream())
    if st != OK:
        raise CovspecError(st, "covspec_stream_step")
    return nxt.value, (c if (want_c and n_keep + p.frame_m > p.keep_k) else None)
