"""Seeded synthetic workloads for the KeyDiff block-prefill path.

This module only *draws inputs*: random keys, queries and values with the
shape and key geometry of the workloads the paper evaluates (Llama / Qwen
layers, block size B, cache budget N; Experiments section, "Experimental
Setup").  It contains none of the method's arithmetic (no attention, no
anchor, no score, no selection), so both the CPU oracle's tests and the HIP
path's tests may import it; it imports neither of them.

All arrays are bf16 *bit patterns* (numpy uint16) so that the very same bits
reach both sides.
"""
from .configs import CONFIGS, Workload, get_config
from .generate import (
    apply_rope,
    bf16_bits_to_f32,
    bf16_bits_to_f64,
    block_of,
    f32_to_bf16_bits,
    make_layer,
    rope_tables,
)

__all__ = [
    "CONFIGS",
    "Workload",
    "get_config",
    "make_layer",
    "rope_tables",
    "apply_rope",
    "block_of",
    "f32_to_bf16_bits",
    "bf16_bits_to_f32",
    "bf16_bits_to_f64",
]
