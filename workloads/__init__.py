"""Seeded synthetic inputs for the TriSpec verification pass.

This package is the only code shared by the CPU oracle's tests and the HIP
path's tests/bench.  It holds no arithmetic of the method itself: it draws
random weights, random KV caches, random tokens and random draft trees, and
rounds stored values to the storage dtype.  Everything is a pure function of
(shape, seed).
"""
from .gen import (  # noqa: F401
    ModelShape,
    SHAPES,
    WeightSource,
    bf16_bits,
    bf16_bits_to_f32,
    gen_context_tokens,
    gen_chain,
    gen_kv_cache,
    gen_tree,
    gen_eagle2_tree,
    gen_draft_tokens,
    gen_draft_distributions,
    gen_uniforms,
    tree_depths,
)
