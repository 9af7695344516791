"""MI355X-native MoE-layer forward path (gate, dispatch, expert FFN, combine, ring offloading).

The compute lives in ``libmoesys_hip.so`` (hand-written HIP for gfx950, C ABI in
``include/moesys.h``); this package only marshals arguments.
"""
from .binding import (  # noqa: F401
    ExpertCache, ExpertPool, MoEConfig, MoEError, Ring, StageTimer, Weights, lib, lib_path,
    moe_capacity, moe_combine, moe_combine_backward, moe_expert_ffn_backward, moe_expert_ffn_backward_workspace_bytes, moe_expert_wgrad, moe_gate_aux_loss, moe_layer_backward, moe_layer_backward_workspace_bytes, moe_dispatch, moe_dispatch_static, moe_expert_ffn, moe_gate, moe_gate_packed, moe_pack_router, moe_router_pack_bytes, moe_layer_forward,
    moe_layer_forward_timed, moe_layer_route, moe_layer_experts, moe_transpose_expert_weights, moe_workspace_bytes, moe_workspace_layout,
    STAGE_NAMES, MOE_TUNE_GEMM_TILE_ROWS, MOE_TUNE_FEW_TOKEN_KERNELS, MOE_TUNE_GATE_TOKENS, MOE_TUNE_GEMM_MFMA, moe_get_tuning, moe_set_tuning,
)
