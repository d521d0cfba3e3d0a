"""Seeded synthetic inputs shared by the fp64 checker and the device path (inputs only)."""
from .gen import (CONFIGS, MARGIN, MoEConfig, bf16_bits, bf16_round, custom_config, expert_weights,
                  layer_inputs, merge_inputs, min_topk_gap, router_bias, to_storage, tokens_with_margin,
                  trainable_mask)

__all__ = ["CONFIGS", "MARGIN", "MoEConfig", "bf16_bits", "bf16_round", "custom_config", "expert_weights",
           "layer_inputs", "merge_inputs", "min_topk_gap", "router_bias", "to_storage", "tokens_with_margin",
           "trainable_mask"]
