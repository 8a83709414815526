"""Seeded synthetic inputs for the sparse-MoE feed-forward layer.

This package only draws random tensors and converts storage formats.  It holds
none of the layer's arithmetic (no logits, softmax, top-k, FFN): the CPU oracle
and the HIP library both receive the arrays made here and nothing else is
shared between them.
"""
from .generate import (  # noqa: F401
    CONFIGS,
    LayerConfig,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    make_inputs,
    make_layer_weights,
    make_stack_weights,
    normal_tensor,
    stored_zipf_bias,
    shrink,
    zipf_target_shares,
)
