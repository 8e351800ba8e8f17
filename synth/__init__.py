"""Seeded synthetic input generators.

This package only manufactures inputs (weights, prompts, planning
vocabularies, logit tables).  It holds none of the decoding method's
arithmetic, so both the CPU oracle's tests and the HIP path's tests can feed
from it without the two sharing any code of the method itself.
"""
from .inputs import (  # noqa: F401
    ModelShape,
    TINY,
    LLADA_8B,
    bf16_round,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    make_weights,
    make_consistent_weights,
    prior_plan_vocab,
    make_prompt,
    make_plan_vocab,
    plan_bitmap,
    make_boosted_logits,
    table_model_logits,
)
