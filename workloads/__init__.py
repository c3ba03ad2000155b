"""Seeded synthetic inputs for the MoE-layer hot path.

This package produces *data only*: layer shapes, random logits, activations,
expert weights and the token-to-rank split.  It contains none of the method's
arithmetic (no routing, no dispatch, no planning), so that both the CPU oracle's
tests and the GPU path's tests/bench can draw identical inputs from it without
sharing any algorithm code.
"""
from .configs import CONFIGS, LayerConfig, get_config  # noqa: F401
from .synth import (  # noqa: F401
    bf16_bits_to_f32,
    expert_weights,
    f32_to_bf16_bits,
    popularity_bias,
    rank_token_offsets,
    ratio_logits,
    step_inputs,
)
