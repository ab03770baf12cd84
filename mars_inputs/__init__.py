"""Seeded synthetic inputs for the MARS verification pass.

This package only draws numbers: logits shaped like the paper's target models
(Vicuna ~32K, LLaMA-3 128 256 and Qwen3 151 936 vocabularies, Sec. 4 / Sec. 5),
EAGLE-style chains and token trees (draft length 7, Sec. 4.1 "Implementation
Details"), draft tokens, uniforms and draft distributions.  It holds none of
the verification arithmetic and is imported by the tests and the benchmark,
which hand the same arrays to the HIP library and to the CPU oracle.
"""
from .generators import (  # noqa: F401
    CONFIGS,
    Workload,
    bf16_bits_to_f32,
    chain_parents,
    f32_to_bf16_bits,
    make_config,
    make_workload,
    random_tree,
)
