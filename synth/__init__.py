"""Seeded synthetic inputs for the draft-block verification step.

This package only *produces numbers* (weights, KV caches, draft tokens and
distributions, uniforms) with the shapes and value distributions of the
paper's Llama-3.1-8B / 70B-shaped workloads.  It holds none of the method's
arithmetic: no transformer math, no accept test, no sampling of the emitted
token.  Both the CPU oracle's tests and the HIP library's tests / benchmark
pull their inputs from here so that the two sides see identical values.
"""
from .configs import CONFIGS, DRAFT_1B, ModelShape, shape_of  # noqa: F401
from .generate import (  # noqa: F401
    bf16_bits_to_f32,
    bf16_bits_to_f64,
    f32_to_bf16_bits,
    WeightSource,
    make_kv_cache,
    make_draft,
    make_prompt,
    make_pending,
    to_f64,
    make_hidden,
    make_judge_dataset,
    TENSOR_NAMES,
)
