"""Seeded synthetic inputs for the token-importance pass.

This package only draws random tensors and integer offset arrays with the
shapes and value distributions of draft-model workloads. It contains none of
the method's arithmetic (no logits, softmax, pooling, selection or projection)
so that both the CPU oracle's tests and the GPU path's tests can feed on it
without sharing any computation.
"""
from .configs import CONFIGS, Workload, get_config
from .gen import (
    SEED,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    gen_char_offsets,
    gen_k_layer,
    gen_look_keys,
    gen_prompt_lengths,
    gen_q,
    heavy_hitter_positions,
    make_score_inputs,
    quantise_k_e4m3,
)

__all__ = [
    "CONFIGS",
    "Workload",
    "get_config",
    "SEED",
    "bf16_bits_to_f32",
    "f32_to_bf16_bits",
    "gen_char_offsets",
    "gen_k_layer",
    "gen_look_keys",
    "gen_prompt_lengths",
    "gen_q",
    "heavy_hitter_positions",
    "make_score_inputs",
    "quantise_k_e4m3",
]
