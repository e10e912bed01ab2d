"""MI355X-native visual token reduction of CoVSpec (paper Sec. III-A) behind a C ABI."""
from .binding import (BF16, FP16, FP32, LR_ENERGY_TOPK, LR_GREEDY_RESIDUAL, LR_RANDOM, LR_SCORE_TOPK, REL_ATTN_SOFTMAX, REL_COSINE_MAX,
                      NUM_STAGE_EVENTS, PROBE_BEGIN, PROBE_END, STAGES, CovspecError, Params, alloc_workspace, load_library, probe_launches, reduce, resolve, score, select,
                      status_string, workspace_size, VerifyParams, verify, verify_static, verify_workspace_size, VERIFY_STATIC_MAX_SCRATCH, DraftParams, draft_fanout, draft_gate, draft_workspace_size, ragged_resolve, ragged_workspace_size, reduce_ragged, lowrank_path, image_status, set_wait_limit_us, StreamParams, stream_alloc_state, stream_step, stream_workspace_size)

__all__ = ["BF16", "FP16", "FP32", "LR_ENERGY_TOPK", "LR_GREEDY_RESIDUAL", "LR_RANDOM", "LR_SCORE_TOPK", "REL_ATTN_SOFTMAX", "REL_COSINE_MAX",
           "NUM_STAGE_EVENTS", "PROBE_BEGIN", "PROBE_END", "STAGES", "CovspecError", "Params", "alloc_workspace", "load_library", "probe_launches", "reduce", "resolve", "score", "select",
           "status_string", "workspace_size", "VerifyParams", "verify", "verify_static", "verify_workspace_size", "VERIFY_STATIC_MAX_SCRATCH", "DraftParams", "draft_fanout", "draft_gate", "draft_workspace_size", "ragged_resolve", "ragged_workspace_size", "reduce_ragged", "lowrank_path", "image_status", "set_wait_limit_us", "StreamParams", "stream_alloc_state", "stream_step", "stream_workspace_size"]
