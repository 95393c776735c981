"""Seeded synthetic inputs for the EntroLLM hot path.

This module draws random numbers and shapes only.  It holds none of the
method's arithmetic (no quantisation, no coding, no dequantisation): both the
CPU oracle's tests and the GPU library's tests and benchmark call it so that
they see the same weights and activation vectors.

The paper evaluates on trained smolLM-1.7B / phi3-mini-4k / mistral-7B weights
(Experiments section); those are not available offline, so every tensor here
is a seeded draw with the same shape and a bell-shaped, heavy-tailed value
distribution that reproduces the "spiky" per-tensor symbol histogram the
Proposed Method section relies on.
"""
from .configs import (  # noqa: F401
    TensorSpec,
    config_tensors,
    config_chunk_symbols,
    config_bits,
    make_tensor,
    make_x_bf16,
    tensor_seed,
    x_seed,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    adversarial_symbol_cases,
)
