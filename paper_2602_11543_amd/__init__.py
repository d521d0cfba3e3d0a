"""SPES MoE-layer hot path for AMD MI355X: thin Python binding over the C-ABI library of HIP kernels."""
from .binding import (SPES_BF16, SPES_F32, SpesError, ctx_view, library_path, moe_shape, spes_expert_merge, spes_expert_pack, spes_upcycle_init,
                      spes_expert_warmup_merge, spes_expert_warmup_merge_static, spes_masked_adamw, spes_moe_bwd, spes_moe_ctx_bytes, spes_moe_ctx_describe, spes_moe_fwd,
                      spes_moe_grad_scatter, spes_moe_permute, spes_moe_router_aux, spes_moe_shape, spes_profile_enable, spes_profile_read, spes_ref_mfma_rate, spes_strerror, spes_warmup_scratch_bytes, torch_dtype)

__all__ = ["SPES_BF16", "SPES_F32", "SpesError", "ctx_view", "library_path", "moe_shape", "spes_expert_merge", "spes_expert_pack", "spes_upcycle_init",
           "spes_expert_warmup_merge", "spes_expert_warmup_merge_static", "spes_masked_adamw", "spes_moe_bwd", "spes_moe_ctx_bytes", "spes_moe_ctx_describe", "spes_moe_fwd",
           "spes_moe_grad_scatter", "spes_moe_permute", "spes_moe_router_aux", "spes_moe_shape", "spes_profile_enable", "spes_profile_read", "spes_ref_mfma_rate", "spes_strerror", "spes_warmup_scratch_bytes", "torch_dtype"]
