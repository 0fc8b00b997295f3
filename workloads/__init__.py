"""Seeded synthetic inputs for the ExpertWeave MoE-layer hot path.

This package serves both the CPU oracle's tests and the HIP path's tests and
benchmark with the *same data*.  It holds no arithmetic of the method itself:
only random draws, dtype rounding/packing, and the shapes of the five
workload configurations.  It imports neither the oracle nor the HIP binding.
"""
from .configs import MoEConfig, CONFIGS, get_config
from .generate import (
    tuned_sets,
    adapter_ids,
    adapter_ids_powerlaw,
    tokens,
    gate_weight,
    expert_weights,
    stacked_expert_weights,
    shared_weights,
    logit_bias_table,
    distinct_topk_ids,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
)

__all__ = [
    "MoEConfig", "CONFIGS", "get_config",
    "tuned_sets", "adapter_ids", "adapter_ids_powerlaw", "tokens", "gate_weight", "expert_weights",
    "stacked_expert_weights", "shared_weights", "logit_bias_table",
    "distinct_topk_ids", "f32_to_bf16_bits", "bf16_bits_to_f32",
]
