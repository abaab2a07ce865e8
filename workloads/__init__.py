"""Seeded synthetic inputs for one Medusa verification step.

This package only *draws inputs* (random tensors, prefix lengths, shape tables).
It contains none of the method's arithmetic: no heads, no tree construction, no
attention, no acceptance.  Both the CPU oracle's tests and the HIP path's
tests/benchmarks import it so that the two sides see byte-identical inputs.
"""
from .configs import CONFIGS, StepConfig, get_config, scaled_config, synthetic_accuracy_table
from .generate import (
    TENSOR_IDS,
    bf16_bits_from_f32,
    f32_from_bf16_bits,
    draw_normal,
    draw_prefix_len,
    make_step_inputs,
)

__all__ = [
    "CONFIGS",
    "StepConfig",
    "get_config",
    "scaled_config",
    "synthetic_accuracy_table",
    "TENSOR_IDS",
    "bf16_bits_from_f32",
    "f32_from_bf16_bits",
    "draw_normal",
    "draw_prefix_len",
    "make_step_inputs",
]
