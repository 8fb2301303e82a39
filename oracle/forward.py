"""Oracle forward passes (numpy, fp64).  Test infrastructure, not the product.

The paper defines the verification pass only as "one parallel forward of the
verifier over the k drafted tokens given the prefix X, returning k+1
next-token distributions" (Sec. 2.1 Eq. 2 for the target, Sec. 3.2 Eq. 5 for
the proxy).  The verifier itself is a standard pre-norm decoder (RMSNorm,
rotary embedding, grouped-query attention, SwiGLU), whose shape the workload
fixes.  Two functions compute it:

* `causal_forward` — the textbook definition: a causal forward over a flat
  token sequence, no cache, no tree.  Used for prefill (to obtain a KV cache)
  and as the brute-force reference the tree pass is pinned to.
* `verify_forward` — the same model over the M tree nodes against a given KV
  cache; node i attends to the whole context and to its ancestors and itself.

shape.qk_norm (an option of the model family the paper evaluates on, not of the paper): queries
and keys pass through an RMSNorm over the head dimension, with weights q_norm / k_norm shared by
all heads of a layer, before the rotary embedding.

Storage modes.  "f32": nothing is rounded (all fp64).  "bf16": what the model
STORES is bf16 — the weights (already rounded by whoever supplies them) and the
KV cache: keys (after the rotary embedding) and values are rounded to bf16
(round-to-nearest-even) where they ENTER the cache, so whatever a pass reads
back from the cache (the context) is rounded, while the tokens of the pass
itself attend to each other with their unrounded keys and values.  Nothing
else is rounded: activations, attention probabilities, sums, norms, rotary
math, softmax and logits stay fp64.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional, Sequence

import numpy as np


# --------------------------------------------------------------------------
# primitives


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round fp64 values to the nearest bf16 (8 significant bits, ties to even),
    returned as fp64.  Single rounding straight from fp64."""
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)  # x = m * 2**e, 0.5 <= |m| < 1
    return np.ldexp(np.rint(np.ldexp(m, 8)), e - 8)


def _identity(x: np.ndarray) -> np.ndarray:
    return x


def rmsnorm(x: np.ndarray, w: np.ndarray, eps: float) -> np.ndarray:
    """x * rsqrt(mean(x^2) + eps) * w over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * w


def rope_angles(positions: np.ndarray, head_dim: int, base: float) -> np.ndarray:
    """angle[p, j] = position_p * base^(-2j/d), j = 0..d/2-1."""
    j = np.arange(head_dim // 2, dtype=np.float64)
    inv_freq = np.power(float(base), -2.0 * j / head_dim)
    return np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]


def apply_rope(t: np.ndarray, angles: np.ndarray) -> np.ndarray:
    """Rotate-half rotary embedding.  t: [T, heads, d]; angles: [T, d/2].
    Pair (j, j + d/2) is rotated by angle j."""
    half = t.shape[-1] // 2
    c = np.cos(angles)[:, None, :]
    s = np.sin(angles)[:, None, :]
    a, b = t[..., :half], t[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def _silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def _softmax(s: np.ndarray) -> np.ndarray:
    e = np.exp(s - np.max(s))
    return e / np.sum(e)


class OracleWeights:
    """Adapter around `get(name, layer) -> array`; hands out fp64 copies."""

    def __init__(self, get: Callable[[str, int], np.ndarray]):
        self._get = get

    def __call__(self, name: str, layer: int = 0) -> np.ndarray:
        return np.asarray(self._get(name, layer), dtype=np.float64)

    def rows(self, name: str, idx) -> np.ndarray:
        """Selected rows of a (large) matrix, e.g. the embeddings of the input tokens."""
        return np.asarray(self._get(name, 0)[np.asarray(idx)], dtype=np.float64)


def _lm_head(h: np.ndarray, W: OracleWeights, vocab: int) -> np.ndarray:
    """logits = h @ Wlm^T.  Rows of Wlm are taken in slabs only to bound memory;
    every logit is still one plain dot product."""
    wl = W._get("lm_head", 0)
    out = np.empty((h.shape[0], vocab), dtype=np.float64)
    slab = 16384
    for lo in range(0, vocab, slab):
        hi = min(vocab, lo + slab)
        out[:, lo:hi] = h @ np.asarray(wl[lo:hi], dtype=np.float64).T
    return out


# --------------------------------------------------------------------------
# textbook causal forward (no cache, no tree)


def causal_forward(W: OracleWeights, shape, tokens: Sequence[int],
                   positions: Optional[Sequence[int]] = None,
                   last_only: bool = False, n_cached: int = 0,
                   in_pass_kv: str = "unrounded") -> Dict[str, np.ndarray]:
    """Plain causal decoder forward over tokens[0..T-1].

    Returns logits [T, V] (or [1, V] for the last row if last_only), and the
    per-layer post-rotary keys / values K, V: [L, n_kv, T, d] as a cache would
    store them (rounded to the storage type).

    n_cached models a cache boundary for the bf16 storage mode: tokens [0, n_cached)
    were processed by an earlier pass, so queries at t >= n_cached see those keys /
    values as the cache holds them (rounded); every other (query, key) pair belongs to
    one pass and uses unrounded values.  With f32 storage it has no effect.

    in_pass_kv = "stored" is the other reading of a bf16 cache: every key / value attention
    reads, the query's own included, is the stored (rounded) one — a decoder that appends to
    its cache before it attends.  n_cached is then immaterial.  (The paper fixes neither; the
    build's reading is "unrounded", and tests bound the difference between the two.)
    """
    if in_pass_kv not in ("unrounded", "stored"):
        raise ValueError(in_pass_kv)
    rnd = bf16_round if shape.dtype == "bf16" else _identity
    T = len(tokens)
    H, nq, nkv, d = shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    group = nq // nkv
    pos = np.arange(T) if positions is None else np.asarray(positions)
    ang = rope_angles(pos, d, shape.rope_base)
    x = W.rows("embed", tokens)
    Ks = np.empty((shape.n_layers, nkv, T, d))
    Vs = np.empty((shape.n_layers, nkv, T, d))
    for l in range(shape.n_layers):
        h = rmsnorm(x, W("norm_attn", l), shape.rms_eps)
        q = (h @ W("wq", l).T).reshape(T, nq, d)
        k = (h @ W("wk", l).T).reshape(T, nkv, d)
        v = (h @ W("wv", l).T).reshape(T, nkv, d)
        if getattr(shape, "qk_norm", False):
            q = rmsnorm(q, W("q_norm", l), shape.rms_eps)
            k = rmsnorm(k, W("k_norm", l), shape.rms_eps)
        q = apply_rope(q, ang)
        k = apply_rope(k, ang)
        Ks[l] = rnd(k).transpose(1, 0, 2)
        Vs[l] = rnd(v).transpose(1, 0, 2)
        o = np.zeros((T, nq, d))
        for t in range(T):
            nc = n_cached if t >= n_cached else 0     # keys this query reads back from the cache
            if in_pass_kv == "stored":
                nc = t + 1
            kt = np.concatenate([rnd(k[:nc]), k[nc: t + 1]], axis=0)
            vt = np.concatenate([rnd(v[:nc]), v[nc: t + 1]], axis=0)
            for a in range(nq):
                g = a // group
                s = (kt[:, g] @ q[t, a]) / np.sqrt(d)
                o[t, a] = _softmax(s) @ vt[:, g]
        x = x + o.reshape(T, nq * d) @ W("wo", l).T
        h = rmsnorm(x, W("norm_ffn", l), shape.rms_eps)
        act = _silu(h @ W("w_gate", l).T) * (h @ W("w_up", l).T)
        x = x + act @ W("w_down", l).T
    if last_only:
        x = x[-1:]
    hf = rmsnorm(x, W("final_norm"), shape.rms_eps)
    return {"logits": _lm_head(hf, W, shape.vocab), "K": Ks, "V": Vs}


def adapter(features: np.ndarray, weight: np.ndarray, bias: Optional[np.ndarray] = None) -> np.ndarray:
    """The one-layer adapter that maps a proxy's features into the feature space the drafter
    expects (Sec. 3.2, "Drafter selection and adapter training"): y = f W^T + b.  The paper states
    neither its shape nor a non-linearity; one affine map [adapter_dim, hidden] is this build's reading."""
    y = np.asarray(features, dtype=np.float64) @ np.asarray(weight, dtype=np.float64).T
    return y if bias is None else y + np.asarray(bias, dtype=np.float64)


# --------------------------------------------------------------------------
# tree-masked verification forward against a KV cache


def ancestor_sets(parents: Sequence[int]) -> List[List[int]]:
    """anc[i] = nodes on the path root..i, inclusive, in root-first order."""
    out: List[List[int]] = []
    for i, p in enumerate(parents):
        if p < 0:
            out.append([i])
        else:
            if not (0 <= p < i):
                raise ValueError("parents must satisfy parents[0] = -1, 0 <= parents[i] < i")
            out.append(out[p] + [i])
    return out


def verify_forward(W: OracleWeights, shape, k_ctx, v_ctx, tokens: Sequence[int],
                   parents: Sequence[int], positions: Sequence[int],
                   keep_hidden: bool = False, trace: Optional[list] = None,
                   in_pass_kv: str = "unrounded") -> Dict[str, np.ndarray]:
    """One verification pass (Eq. 2 / Eq. 5): the M tree nodes against a cache.

    k_ctx, v_ctx: either arrays [L, n_kv, C, d] or callables layer -> [n_kv, C, d]
    (post-rotary keys, values of the C context tokens).
    Node i attends to every context key and to the keys of its ancestors and itself.

    Returns logits [M, V]; k_new, v_new [L, n_kv, M, d] (what the pass appends to
    the cache at slots C..C+M-1, rounded to the storage type; the nodes themselves attend
    to each other with the unrounded values); optionally the per-layer residual stream.  If `trace`
    is a list, one dict of intermediates per layer is appended to it (q, k, v as fed to
    attention, the unrounded attention output o, the residual stream after attention and
    after the FFN, the SiLU(gate)*up product).
    in_pass_kv = "stored": the nodes attend to each other with the stored (rounded) keys and
    values as well — the other reading of a bf16 cache, see causal_forward.
    """
    if in_pass_kv not in ("unrounded", "stored"):
        raise ValueError(in_pass_kv)
    rnd = bf16_round if shape.dtype == "bf16" else _identity
    M = len(tokens)
    H, nq, nkv, d = shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    group = nq // nkv
    anc = ancestor_sets(parents)
    ang = rope_angles(np.asarray(positions), d, shape.rope_base)
    x = W.rows("embed", tokens)
    k_new = np.empty((shape.n_layers, nkv, M, d))
    v_new = np.empty((shape.n_layers, nkv, M, d))
    hidden = []
    for l in range(shape.n_layers):
        kc = np.asarray(k_ctx(l) if callable(k_ctx) else k_ctx[l], dtype=np.float64)
        vc = np.asarray(v_ctx(l) if callable(v_ctx) else v_ctx[l], dtype=np.float64)
        h = rmsnorm(x, W("norm_attn", l), shape.rms_eps)
        q = (h @ W("wq", l).T).reshape(M, nq, d)
        k = (h @ W("wk", l).T).reshape(M, nkv, d)
        v = (h @ W("wv", l).T).reshape(M, nkv, d)
        if getattr(shape, "qk_norm", False):
            q = rmsnorm(q, W("q_norm", l), shape.rms_eps)
            k = rmsnorm(k, W("k_norm", l), shape.rms_eps)
        q = apply_rope(q, ang)
        k = apply_rope(k, ang)
        k_new[l] = rnd(k).transpose(1, 0, 2)      # what enters the cache
        v_new[l] = rnd(v).transpose(1, 0, 2)
        kd, vd = (rnd(k), rnd(v)) if in_pass_kv == "stored" else (k, v)   # what the nodes see of each other
        o = np.zeros((M, nq, d))
        for i in range(M):
            for a in range(nq):
                g = a // group
                keys = np.concatenate([kc[g], kd[anc[i], g]], axis=0)
                vals = np.concatenate([vc[g], vd[anc[i], g]], axis=0)
                s = (keys @ q[i, a]) / np.sqrt(d)
                o[i, a] = _softmax(s) @ vals
        x = x + o.reshape(M, nq * d) @ W("wo", l).T
        x_mid = x
        h = rmsnorm(x, W("norm_ffn", l), shape.rms_eps)
        act = _silu(h @ W("w_gate", l).T) * (h @ W("w_up", l).T)
        x = x + act @ W("w_down", l).T
        if trace is not None:
            trace.append({"q": q, "k": k, "v": v, "o": o.reshape(M, nq * d), "x_mid": x_mid,
                          "act": act, "x": x})
        if keep_hidden:
            hidden.append(x.copy())
    hf = rmsnorm(x, W("final_norm"), shape.rms_eps)
    out = {"logits": _lm_head(hf, W, shape.vocab), "k_new": k_new, "v_new": v_new,
           "final_hidden": hf}
    if keep_hidden:
        out["hidden"] = np.stack(hidden)
    return out
