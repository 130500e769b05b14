"""Seeded synthetic MoE-layer inputs.

This package only draws random numbers and rounds them to their storage
precision. It holds none of the MoE layer's arithmetic, and both the CPU
oracle's tests and the GPU path's tests/bench take their inputs from it.
"""
from .synth import (  # noqa: F401
    LayerConfig,
    CONFIGS,
    mixtral_sweep_config,
    f32_to_bf16_bits,
    make_activations,
    make_logits,
    make_router_weight,
    make_expert_weights,
    make_all_expert_weights,
    zipf_bias,
    MIXTRAL_SWEEP_T,
    microbatch_ranges,
)
