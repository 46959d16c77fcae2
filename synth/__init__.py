"""Seeded synthetic inputs (weights, KV fill, hidden states, prompts).

This module is the only code shared by the CPU oracle and the HIP path.  It
produces bytes; it contains none of the method's arithmetic (no norm, RoPE,
attention, GEMM, argmax, block layout or n-gram logic).
"""
from .gen import (  # noqa: F401
    ModelShape,
    SHAPES,
    bf16_bits,
    bf16_to_f32,
    layer_weights,
    head_weights,
    normal,
    kv_fill,
    hidden_block,
    uniform_prompt,
    markov_prompt,
)
