"""Seeded synthetic inputs for the MoE-layer hot path.

This package is shared by the CPU oracle's tests and by the HIP path's tests
and benchmark.  It only draws random tensors and rounds them to the storage
type; it holds none of the layer's arithmetic (no router product, no softmax,
no top-k, no permutation, no expert FFN).
"""
from .configs import CONFIGS, LayerConfig, get_config
from .generate import (
    LayerInputs,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    make_layer_inputs,
    make_logits,
    make_tokens,
    redraw_token_rows,
)

__all__ = [
    "CONFIGS",
    "LayerConfig",
    "get_config",
    "LayerInputs",
    "bf16_bits_to_f32",
    "f32_to_bf16_bits",
    "make_layer_inputs",
    "make_logits",
    "make_tokens",
    "redraw_token_rows",
]
