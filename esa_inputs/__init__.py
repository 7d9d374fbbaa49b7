"""Seeded synthetic inputs for Efficient Selective Attention (ESA) workloads.

This package only manufactures data: normal draws from a counter-based
generator, rotary position encoding of the raw queries/keys, seeded linear
compression weights, and the planted structure (needle keys, pushed-down keys).  It
contains none of the method's arithmetic (no compression of activations, no
scoring, no selection, no attention), so both the CPU oracle's tests and the
HIP path's harness may draw their inputs from it.
"""
from .configs import EsaConfig, CONFIGS, get_config, segment_bounds, chunk_starts
from .generate import (
    LayerInputs,
    make_layer,
    make_weights,
    needle_plan,
    push_keys_down,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    storage_to_f64,
)

__all__ = [
    "EsaConfig", "CONFIGS", "get_config", "segment_bounds", "chunk_starts",
    "LayerInputs", "make_layer", "make_weights", "needle_plan", "push_keys_down",
    "f32_to_bf16_bits", "bf16_bits_to_f32", "storage_to_f64",
]
