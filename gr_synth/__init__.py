"""Seeded synthetic inputs for the generative-recommendation decode step.

This module only *draws data*: beam queries, prompt / decode K and V, per-step logits, prompt
lengths and the sorted table of valid semantic-ID tuples.  It contains none of the method's
arithmetic (no attention, no masking, no log-softmax, no selection) and is the single piece of code
that both the CPU oracle's tests and the GPU path's tests and benchmark are allowed to share.

Shapes and distributions follow the paper's workload description: three tokens per item
(Section 2.2.1), beam widths of 128-512 (Sections 2.2.1, 9.1), prompts of hundreds to thousands
of tokens (Section 1), thousands of valid first-step tokens and few valid last-step tokens
(Section 6.1).  The paper's datasets and trained weights are not available, so every value is
random: Q/K/V ~ N(0,1) rounded to bf16, logits ~ sigma * N(0,1) in fp32.
"""
from .configs import CONFIGS, GRConfig, get_config
from .generate import (
    bf16_bits_to_f32,
    e4m3_bits_to_f32,
    f32_to_bf16_bits,
    f32_to_e4m3_bits,
    initial_beam_state,
    make_attention_inputs,
    make_item_table,
    make_logits,
    make_prompt_lengths,
    rng_for,
)

__all__ = [
    "CONFIGS", "GRConfig", "get_config", "bf16_bits_to_f32", "f32_to_bf16_bits", "e4m3_bits_to_f32", "f32_to_e4m3_bits",
    "initial_beam_state", "make_attention_inputs", "make_item_table", "make_logits",
    "make_prompt_lengths", "rng_for",
]
