"""UniPool shared-pool MoE layer for MI355X: Python binding over the C-ABI library."""
from .binding import (  # noqa: F401
    BF16, F32, ROUTER_NORM, ROUTER_SOFTMAX, Shape, UniPoolError, combine, combine_bwd, distinct_experts, estimate_c, expert_ffn_bwd, expert_ffn_fwd, expert_ffn_fwd_gather, expert_ffn_recompute,
    expert_wgrad, fast_path, last_error, lib_path, load_library, permute, permute_static, pool_aux_loss, route, route_bwd,
    version, workspace_bytes,
)
