"""Expert-choice MoE layer for MI355X: thin Python binding over libec_moe.so.

The package only marshals arguments; every step of the layer runs in the HIP
kernels behind the C ABI declared in include/ec_moe.h.  There is no CPU or
PyTorch fallback: a missing library is an error.
"""
from .binding import (  # noqa: F401
    EC_ACT_GELU, EC_ACT_IDENTITY, EC_ACT_RELU, EC_BF16, EC_BF16_HILO, EC_F32, EC_MOE_MAX_EXPERTS,
    EcMoeError, alloc_workspace, ec_moe_backward, ec_moe_backward_timed, ec_moe_capacity, ec_moe_capped_assignment,
    ec_moe_capped_workspace_bytes, ec_moe_forward_capped, ec_moe_combine, ec_moe_combine_static, ec_moe_dispatch,
    ec_moe_expert_ffn, ec_moe_forward, ec_moe_forward_grouped, ec_moe_forward_token_choice, ec_moe_gate, ec_moe_last_hip_error, ec_moe_status_string,
    ec_moe_token_choice, ec_moe_topk_tokens, ec_moe_topk_tokens_grouped, ec_moe_version, ec_moe_workspace_bytes, lib, lib_path,
)
