"""MI355X-native MoE expert layer (the hot path Fiddler, arXiv 2402.07033,
schedules): thin Python binding over the C ABI of libmoe_hip.so.

Every step runs in hand-written HIP kernels; PyTorch only provides device
memory and streams.  There is no CPU fallback: importing the binding's
functions without the built library raises.
"""
from .binding import (ORCH_CPU, ORCH_GPU_RESIDENT, ORCH_GPU_TRANSFER, ORCH_SKIP, OrchLayer,
                      moe_orch_cpu_expert_ffn, moe_orch_decide, moe_orch_hit_rate, moe_orch_place,
                      MOE_BF16, MOE_F32, MOE_FFN_AUTO, MOE_FFN_GROUPED, MOE_FFN_MID,
                      MOE_FFN_STREAM, MoeError, PackedWeights, StackBuffers, lib, lib_path,
                      moe_combine, moe_combine_norm_route_permute, moe_combine_parts,
                      moe_combine_residual, moe_decode_block, moe_decode_block_supported, moe_decode_layer, moe_expert_ffn,
                      moe_expert_ffn_noalloc, moe_expert_ffn_noalloc_max_bytes,
                      moe_expert_ffn_parts, moe_expert_ffn_plan, moe_expert_ffn_tokens, moe_expert_ffn_workspace,
                      moe_hbm_read_probe, moe_layer, moe_mfma_rate_probe,
                      moe_norm_route_permute, moe_permute, moe_residual_add, moe_rmsnorm,
                      moe_gate_sums, moe_gate_sums_stride, moe_rmsnorm_router_logits, moe_route, moe_route_permute,
                      moe_router_logits, moe_set_ffn_mid_event, moe_stack_forward,
                      moe_status_string, moe_weights_free, moe_weights_pack)

__all__ = [
    "ORCH_CPU", "ORCH_GPU_RESIDENT", "ORCH_GPU_TRANSFER", "ORCH_SKIP", "OrchLayer",
    "moe_orch_cpu_expert_ffn", "moe_orch_decide", "moe_orch_hit_rate", "moe_orch_place",
    "MOE_BF16", "MOE_F32", "MOE_FFN_AUTO", "MOE_FFN_GROUPED", "MOE_FFN_MID", "MOE_FFN_STREAM",
    "MoeError", "PackedWeights", "StackBuffers", "lib", "lib_path", "moe_combine",
    "moe_combine_norm_route_permute", "moe_combine_parts", "moe_combine_residual",
    "moe_decode_block", "moe_decode_block_supported", "moe_decode_layer", "moe_expert_ffn", "moe_expert_ffn_noalloc",
    "moe_expert_ffn_noalloc_max_bytes", "moe_expert_ffn_parts", "moe_expert_ffn_tokens", "moe_expert_ffn_plan",
    "moe_expert_ffn_workspace", "moe_hbm_read_probe", "moe_layer", "moe_mfma_rate_probe",
    "moe_norm_route_permute", "moe_permute", "moe_residual_add", "moe_rmsnorm",
    "moe_gate_sums", "moe_gate_sums_stride", "moe_rmsnorm_router_logits", "moe_route", "moe_route_permute", "moe_router_logits",
    "moe_set_ffn_mid_event", "moe_stack_forward", "moe_status_string", "moe_weights_free",
    "moe_weights_pack",
]
