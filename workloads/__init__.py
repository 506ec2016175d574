"""Seeded synthetic input generators for the tree-verification workloads.

This package only draws inputs (trees, Q/K/V tensors, logits, draft
distributions, tokens, uniforms).  It contains none of the arithmetic of the
verification method itself and is the one module shared by the CPU oracle's
tests and the HIP path's tests and benchmark.
"""
from .generators import (  # noqa: F401
    CONFIGS,
    VerifyConfig,
    accept_inputs,
    attention_inputs,
    bf16_bits,
    bf16_bits_to_f32,
    chain_tree,
    coin_tree,
    config_rng,
    draft_head_inputs,
    moe_inputs,
    paged_layout,
    round_to_bf16,
    static_tree,
    tree_depths,
    two_expert_tree,
    tree_for_config,
)
