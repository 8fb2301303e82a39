"""Shared test helpers (no method arithmetic): shape shorthands and oracle drivers."""
import numpy as np

from oracle import OracleWeights, causal_forward, verify_forward
from workloads import ModelShape, WeightSource, gen_context_tokens, tree_depths

MICRO = ModelShape("micro", 2, 32, 4, 2, 8, 48, 61, "f32", rope_base=1e4, lm_head_std=0.8)


def oracle_weights(shape, seed):
    return OracleWeights(WeightSource(shape, seed).get)


def prefill(shape, seed, ctx_tokens, start_pos=0):
    """Oracle KV cache of the context (post-rotary K, V): [L, n_kv, C, d]."""
    W = oracle_weights(shape, seed)
    if len(ctx_tokens) == 0:
        z = np.zeros((shape.n_layers, shape.n_kv_heads, 0, shape.head_dim))
        return z, z.copy()
    out = causal_forward(W, shape, ctx_tokens, positions=start_pos + np.arange(len(ctx_tokens)),
                         last_only=True)
    return out["K"], out["V"]


def path_to(parents, i):
    p = []
    while i >= 0:
        p.append(i)
        i = parents[i]
    return p[::-1]
