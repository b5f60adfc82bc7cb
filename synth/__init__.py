"""Seeded synthetic inputs for the DualSparse-MoE layer (shared by the oracle tests and the GPU path).

This package holds no arithmetic of the method itself: it only draws random tensors of the
shapes and value distributions of the benchmark layers, rounds them to bf16 where asked, and
describes the layer configurations.  It imports neither the oracle nor the GPU binding.
"""
from .layers import (  # noqa: F401
    LayerSpec,
    LAYERS,
    make_layer,
    make_logits,
    make_perm,
    make_router,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    zipf_logit_bias,
)
