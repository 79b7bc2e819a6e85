"""Seeded synthetic inputs (model shapes, weights, prompts, KV fills, draws).

This package serves both the CPU oracle and the HIP path.  It holds no arithmetic of
the decoding method itself: only shapes, random draws and the bf16 storage format of
the canonical weights.
"""
from .synthetic import (  # noqa: F401
    ModelShape,
    SHAPES,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    layer_weights,
    head_weights,
    all_weights,
    prompt_tokens,
    normal_bf16,
    ragged_context_lengths,
    geometric_accept_lengths,
)
