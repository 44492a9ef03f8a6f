"""MI355X-native MoE verification layer (router top-k, permute, grouped SwiGLU, combine,
greedy acceptance) as a C-ABI HIP library with a thin ctypes binding."""
from .binding import (  # noqa: F401
    SpecMoEError, lib_path, load_library, moe_combine, moe_expert_down, moe_expert_up_swiglu, moe_expert_up_swiglu_gather, moe_grouped_swiglu,
    moe_grouped_swiglu_static, moe_pack_weights, moe_packed_h_bytes,
    moe_expert_up_swiglu_gather_packed, moe_expert_down_packed,
    moe_permute_rows_packed, moe_expert_up_swiglu_packed,
    moe_grouped_swiglu_workspace_bytes, moe_hot_experts, moe_permute, moe_rmsnorm, moe_route_topk, spec_accept,
    status_string, EXPORTED_SYMBOLS,
    moe_affinity_table, moe_affinity_table_workspace_bytes, moe_nearest_draft_expert,
    moe_route_topk_draft, spec_accept_sample, spec_greedy_tokens, moe_active_expert_bytes,
)
from .layer import GraphedStep, MoEVerifyLayer, MoEVerifyStack  # noqa: F401
