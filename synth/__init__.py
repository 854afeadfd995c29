"""Seeded synthetic inputs for the MoE draft/verify layer.

This package only *generates inputs*: layer shapes, random weights and activations,
router-logit biases that give the requested expert popularity, and the round-to-nearest
group quantiser that turns bf16 expert weights into (code, scale, zero) triples.  It holds
none of the layer's own arithmetic (no routing, no dequantisation, no FFN) and is imported
by both the CPU oracle's tests and the GPU path's tests and benchmark, so that the two
sides see bit-identical inputs.
"""
from .configs import LayerConfig, CONFIGS, config_by_name
from .gen import (
    make_router,
    make_experts_bf16,
    quantize_rtn_int4,
    quantize_rtn_int4_symmetric,
    make_tokens,
    make_layer,
    zipf_bias,
    skew_bias,
    layer_seed,
)

__all__ = [
    "LayerConfig", "CONFIGS", "config_by_name",
    "make_router", "make_experts_bf16", "quantize_rtn_int4",
    "quantize_rtn_int4_symmetric", "make_tokens", "make_layer",
    "zipf_bias", "skew_bias", "layer_seed",
]
