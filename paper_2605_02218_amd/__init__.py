"""MI355X-native visual token reduction of CoVSpec (paper Sec. III-A) behind a C ABI."""
from .binding import (BF16, FP32, LR_ENERGY_TOPK, LR_GREEDY_RESIDUAL, REL_ATTN_SOFTMAX, REL_COSINE_MAX,
                      JACOBI_MAX_SWEEPS, NUM_STAGE_EVENTS, STAGES, CovspecError, Params, alloc_workspace, load_library, reduce, resolve, score, select,
                      status_string, workspace_size)

__all__ = ["BF16", "FP32", "LR_ENERGY_TOPK", "LR_GREEDY_RESIDUAL", "REL_ATTN_SOFTMAX", "REL_COSINE_MAX",
           "JACOBI_MAX_SWEEPS", "NUM_STAGE_EVENTS", "STAGES", "CovspecError", "Params", "alloc_workspace", "load_library", "reduce", "resolve", "score", "select",
           "status_string", "workspace_size"]
