"""Seeded synthetic KV-cache inputs.

Data only: this package holds none of the compression method's arithmetic.  Both
the CPU oracle's tests and the GPU path's tests/bench draw their inputs from
here, so the two sides read exactly the same stored bits.
"""
from .configs import CONFIGS, KVConfig, get_config
from .generate import (
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    generate_sequence,
    generate_unit,
    layer_outlier_positions,
)

__all__ = [
    "CONFIGS",
    "KVConfig",
    "get_config",
    "generate_sequence",
    "generate_unit",
    "layer_outlier_positions",
    "f32_to_bf16_bits",
    "bf16_bits_to_f32",
]
