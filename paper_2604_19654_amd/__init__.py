"""MI355X-native single-rank MoE hot path of FEPLB: a thin ctypes binding over
libfeplb.so (hand-written HIP kernels behind a C ABI, see include/feplb.h)."""
from .binding import (  # noqa: F401
    FeplbError, Group, Move, ORD_MAX, F32, BF16, FFN_GATE_UP, FFN_DOWN, FFN_SCHEDULE, FFN_ALL,
    PLAN_WHOLE, PLAN_OVERFLOW, lib, lib_path, version, HipEvent,
    feplb_route_topk, feplb_permute, feplb_permute_workspace_bytes,
    feplb_grouped_ffn, feplb_grouped_ffn_workspace_bytes, feplb_grouped_ffn_static, STATIC_WS_BYTES,
    feplb_unpermute_combine, feplb_stage_weights, feplb_stream_wait,
    feplb_expert_bytes, feplb_plan,
    BWD_SCHEDULE, BWD_TRANSPOSE, BWD_DGRAD, BWD_WGRAD, BWD_ALL, BWD_ACCUMULATE,
    feplb_grouped_ffn_backward, feplb_grouped_ffn_backward_wt_bytes,
    feplb_combine_backward, feplb_route_topk_backward,
    feplb_history_update, feplb_place, feplb_mark_dynamic, feplb_apply_moves, feplb_straggler, HIST_FRAC_BITS,
)
from .layer import RankLayer, LayerBuffers  # noqa: F401
