"""Seeded generators: model shapes, weights, KV caches, tokens, draft trees.

The paper evaluates on trained Qwen3 / DeepSeek-R1-Distill checkpoints and
public benchmarks (Sec. 4.1); none of them is available here and the latency
of a verification pass does not depend on token values, so every input is
synthetic and a pure function of (shape, seed):

* weights ~ N(0, 0.02^2); the LM head ~ N(0, lm_head_std^2) with a per-shape
  constant that spreads the top-1 probabilities over (0.05, 0.99);
  norm weights ~ 1 + 0.1 N(0,1) (not all-ones, so a kernel that drops or
  mixes up a norm weight fails parity);
* KV caches ~ N(0,1) for the large shapes (a real prefill of thousands of
  tokens through a billion-parameter model is not affordable on the CPU);
* context tokens and draft tokens uniform on [0, V);
* draft trees: a spine to the maximum depth plus random attachments, or an
  EAGLE-2-shaped tree (depth 6, up to 10 children, 60 nodes; paper Sec. 4.1).

Values are rounded to the storage dtype here (bf16 round-to-nearest-even), so
both consumers see the same bytes.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Dict, List, Tuple

import numpy as np

# --------------------------------------------------------------------------
# shapes


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    dtype: str  # "f32" | "bf16"
    rms_eps: float = 1e-6
    rope_base: float = 1e4
    lm_head_std: float = 0.02  # std of the LM-head entries
    qk_norm: bool = False      # per-head RMSNorm of queries and keys before the rotary embedding (Qwen3)

    def with_(self, **kw) -> "ModelShape":
        return replace(self, **kw)

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    def weight_bytes(self) -> int:
        w = 4 if self.dtype == "f32" else 2
        per_layer = (2 * self.hidden * self.q_dim + 2 * self.hidden * self.kv_dim
                     + 3 * self.hidden * self.ffn + 2 * self.hidden)
        return (self.n_layers * per_layer + self.vocab * self.hidden) * w


# lm_head_std = s / sqrt(hidden): the final norm output has RMS ~1, so logits
# have std ~s.  s was picked per vocabulary size so that the oracle's per-node
# top-1 probability covers roughly 0.05..0.99 over seeds (s = 6.5 at V = 4096,
# s = 9.5 at V ~ 1.5e5: median top-1 about 0.5, 10%..90% quantiles about 0.25..0.9).
SHAPES: Dict[str, ModelShape] = {
    # workload 1: tiny fp32 decoder
    "tiny": ModelShape("tiny", 2, 256, 4, 2, 64, 512, 4096, "f32",
                       rope_base=1e4, lm_head_std=6.5 / 16.0),
    # same shape in bf16 storage (exercises the MFMA path at oracle-friendly size)
    "tiny_bf16": ModelShape("tiny_bf16", 2, 256, 4, 2, 128, 512, 4096, "bf16",
                            rope_base=1e4, lm_head_std=6.5 / 16.0),
    # workload 2: Qwen3-0.6B-shaped proxy
    "qwen3_0p6b": ModelShape("qwen3_0p6b", 28, 1024, 16, 8, 128, 3072, 151936, "bf16",
                             rope_base=1e6, lm_head_std=9.5 / 32.0),
    # workload 4, proxy: Qwen3-1.7B-shaped
    "qwen3_1p7b": ModelShape("qwen3_1p7b", 28, 2048, 16, 8, 128, 6144, 151936, "bf16",
                             rope_base=1e6, lm_head_std=9.5 / 45.254833995939045),
    # workload 3 and workload 4's target: Qwen3-8B-shaped
    "qwen3_8b": ModelShape("qwen3_8b", 36, 4096, 32, 8, 128, 12288, 151936, "bf16",
                           rope_base=1e6, lm_head_std=9.5 / 64.0),
    # workload 5: LLaMA-3-8B-shaped
    "llama3_8b": ModelShape("llama3_8b", 32, 4096, 32, 8, 128, 14336, 128256, "bf16",
                            rope_base=5e5, lm_head_std=9.5 / 64.0),
}

# --------------------------------------------------------------------------
# storage rounding


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even. No NaNs expected."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> the float32 values they denote (exact)."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# random numbers: one Philox stream per (seed, tensor id, chunk)

_CHUNK = 1 << 22  # elements per independently seeded chunk


def _n_threads() -> int:
    try:
        return max(1, min(16, int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1)))
    except ValueError:
        return max(1, min(16, os.cpu_count() or 1))


def _normal(seed: int, tensor_id: int, n: int) -> np.ndarray:
    """n standard normals (float32), reproducible regardless of thread count."""
    out = np.empty(n, dtype=np.float32)
    n_chunks = (n + _CHUNK - 1) // _CHUNK

    def fill(c: int) -> None:
        lo = c * _CHUNK
        hi = min(n, lo + _CHUNK)
        g = np.random.Generator(np.random.Philox(key=[seed, tensor_id], counter=[0, 0, c, 0]))
        g.standard_normal(hi - lo, dtype=np.float32, out=out[lo:hi])

    if n_chunks <= 1:
        for c in range(n_chunks):
            fill(c)
    else:
        with ThreadPoolExecutor(_n_threads()) as ex:
            list(ex.map(fill, range(n_chunks)))
    return out


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


# tensor ids
_T_EMBED, _T_LMHEAD, _T_FNORM = 0, 1, 2
_LAYER_BASE, _LAYER_STRIDE = 16, 16
_LAYER_TENSORS = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_ffn", "q_norm", "k_norm")
_T_KV = 1 << 20  # KV-cache streams start here


class WeightSource:
    """Lazily generated weights of one model.

    `get(name, layer)` returns the tensor as float32 holding exactly the values
    stored (already rounded to bf16 when shape.dtype == "bf16"); `bits(...)`
    returns the bf16 bit patterns for upload.  Nothing is cached: a consumer
    that needs a tensor twice asks twice (the 8B shapes do not fit in host
    memory as float32 all at once).
    """

    def __init__(self, shape: ModelShape, seed: int):
        self.shape = shape
        self.seed = int(seed)

    def dims(self, name: str) -> Tuple[int, ...]:
        s = self.shape
        return {
            "embed": (s.vocab, s.hidden),
            "lm_head": (s.vocab, s.hidden),
            "final_norm": (s.hidden,),
            "wq": (s.q_dim, s.hidden),
            "wk": (s.kv_dim, s.hidden),
            "wv": (s.kv_dim, s.hidden),
            "wo": (s.hidden, s.q_dim),
            "w_gate": (s.ffn, s.hidden),
            "w_up": (s.ffn, s.hidden),
            "w_down": (s.hidden, s.ffn),
            "norm_attn": (s.hidden,),
            "norm_ffn": (s.hidden,),
            "q_norm": (s.head_dim,),
            "k_norm": (s.head_dim,),
        }[name]

    def _tensor_id(self, name: str, layer: int) -> int:
        if name == "embed":
            return _T_EMBED
        if name == "lm_head":
            return _T_LMHEAD
        if name == "final_norm":
            return _T_FNORM
        return _LAYER_BASE + _LAYER_STRIDE * layer + _LAYER_TENSORS.index(name)

    def _raw(self, name: str, layer: int) -> np.ndarray:
        dims = self.dims(name)
        n = int(np.prod(dims))
        z = _normal(self.seed, self._tensor_id(name, layer), n)
        if name in ("final_norm", "norm_attn", "norm_ffn", "q_norm", "k_norm"):
            z *= np.float32(0.1)
            z += np.float32(1.0)
        elif name == "lm_head":
            z *= np.float32(self.shape.lm_head_std)
        else:
            z *= np.float32(0.02)
        return z.reshape(dims)

    def get(self, name: str, layer: int = 0) -> np.ndarray:
        z = self._raw(name, layer)
        if self.shape.dtype == "bf16":
            return bf16_bits_to_f32(bf16_bits(z))
        return z

    def bits(self, name: str, layer: int = 0) -> np.ndarray:
        assert self.shape.dtype == "bf16"
        return bf16_bits(self._raw(name, layer))

    def rows(self, name: str, layer: int, row_idx: np.ndarray) -> np.ndarray:
        """Selected rows of a tensor (float32 values as stored)."""
        return self.get(name, layer)[np.asarray(row_idx)]


# --------------------------------------------------------------------------
# tokens, KV, trees


def gen_context_tokens(vocab: int, n: int, seed: int) -> np.ndarray:
    return _rng(seed, 101).integers(0, vocab, size=n, dtype=np.int64).astype(np.int32)


def gen_kv_cache(shape: ModelShape, batch: int, ctx_len: int, seed: int, layer: int):
    """Synthetic post-RoPE K and V of one layer: [batch, n_kv, ctx_len, d] ~ N(0,1),
    float32 values as stored (bf16-rounded for bf16 shapes)."""
    n = batch * shape.n_kv_heads * ctx_len * shape.head_dim
    dims = (batch, shape.n_kv_heads, ctx_len, shape.head_dim)
    k = _normal(seed, _T_KV + 2 * layer, n).reshape(dims)
    v = _normal(seed, _T_KV + 2 * layer + 1, n).reshape(dims)
    if shape.dtype == "bf16":
        k = bf16_bits_to_f32(bf16_bits(k))
        v = bf16_bits_to_f32(bf16_bits(v))
    return k, v


def gen_chain(n_nodes: int) -> np.ndarray:
    """parents of a linear chain: root 0, node i hangs under i-1."""
    return np.arange(-1, n_nodes - 1, dtype=np.int32)


def tree_depths(parents: np.ndarray) -> np.ndarray:
    d = np.zeros(len(parents), dtype=np.int32)
    for i in range(1, len(parents)):
        d[i] = d[parents[i]] + 1
    return d


def _level_order(parents: List[int]) -> np.ndarray:
    """Relabel so that nodes are sorted by depth (stable), parents[i] < i."""
    n = len(parents)
    depth = [0] * n
    for i in range(1, n):
        depth[i] = depth[parents[i]] + 1
    order = sorted(range(n), key=lambda i: (depth[i], i))
    new_id = {old: new for new, old in enumerate(order)}
    out = np.empty(n, dtype=np.int32)
    for old in range(n):
        out[new_id[old]] = -1 if parents[old] < 0 else new_id[parents[old]]
    return out


def gen_tree(n_nodes: int, max_depth: int, max_children: int, seed: int) -> np.ndarray:
    """Random draft tree: a spine root->depth max_depth, then every further node hangs
    under a uniformly chosen node that still has room (depth < max_depth and fewer than
    max_children children).  Returned in level order."""
    assert n_nodes >= 1
    g = _rng(seed, 202)
    parents = [-1]
    depth = [0]
    kids = [0]
    spine = min(max_depth, n_nodes - 1)
    for i in range(1, spine + 1):
        parents.append(i - 1)
        depth.append(i)
        kids.append(0)
        kids[i - 1] += 1
    while len(parents) < n_nodes:
        room = [i for i in range(len(parents)) if depth[i] < max_depth and kids[i] < max_children]
        if not room:
            raise ValueError("tree budget does not fit depth/branching limits")
        p = room[int(g.integers(0, len(room)))]
        parents.append(p)
        depth.append(depth[p] + 1)
        kids.append(0)
        kids[p] += 1
    return _level_order(parents)


def gen_eagle2_tree(seed: int, n_nodes: int = 60, depth: int = 6, top_k: int = 10) -> np.ndarray:
    """EAGLE-2-shaped tree (paper Sec. 4.1: depth 6, expansion top-k 10, 60 tokens):
    the root gets top_k children; every deeper level gets top_k nodes spread at random
    over the previous level (at most top_k per parent); trimmed to n_nodes."""
    g = _rng(seed, 203)
    parents = [-1]
    level = [0]
    for _ in range(depth):
        nxt = []
        counts = {p: 0 for p in level}
        for _ in range(top_k):
            if len(parents) >= n_nodes:
                break
            room = [p for p in level if counts[p] < top_k]
            p = room[int(g.integers(0, len(room)))]
            counts[p] += 1
            parents.append(p)
            nxt.append(len(parents) - 1)
        if not nxt:
            break
        level = nxt
    return _level_order(parents)


def gen_draft_tokens(parents: np.ndarray, vocab: int, seed: int) -> np.ndarray:
    """Uniform random token per node; siblings get distinct tokens."""
    g = _rng(seed, 303)
    n = len(parents)
    tok = np.empty(n, dtype=np.int32)
    used: Dict[int, set] = {}
    for i in range(n):
        s = used.setdefault(int(parents[i]), set())
        while True:
            t = int(g.integers(0, vocab))
            if t not in s:
                break
        s.add(t)
        tok[i] = t
    return tok


# ---------------------------------------------------------------- sampling-mode inputs
def gen_draft_distributions(verifier_logits: np.ndarray, temperature: float, seed: int, noise: float = 0.7,
                            keep: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """A stand-in drafter for a chain of M nodes whose verifier logits are given ([M, V]): its
    distribution at node i is softmax((l_i + noise * N(0,1)) / T) — close to the verifier's, so
    acceptance is neither certain nor hopeless — optionally cut to its `keep` most probable
    tokens and renormalised (a drafter with a reduced vocabulary gives zero mass elsewhere).
    Node i + 1's token is drawn from row i; node 0's token is uniform.
    Returns (p_draft [M-1, V] float32, tokens [M] int32)."""
    g = _rng(seed, 404)
    l = np.asarray(verifier_logits, dtype=np.float64)
    M, V = l.shape
    tokens = np.empty(M, dtype=np.int32)
    tokens[0] = int(g.integers(0, V))
    p_draft = np.zeros((max(M - 1, 0), V), dtype=np.float32)
    for i in range(M - 1):
        z = (l[i] + noise * g.standard_normal(V)) / temperature
        e = np.exp(z - z.max())
        if keep and keep < V:
            e[np.argsort(e)[: V - keep]] = 0.0
        q = (e / e.sum()).astype(np.float32)
        p_draft[i] = q
        c = np.cumsum(q.astype(np.float64))
        tokens[i + 1] = min(int(np.searchsorted(c, g.random() * c[-1], side="right")), V - 1)
    return p_draft, tokens


def gen_uniforms(seed: int, batch: int, n_nodes: int) -> Tuple[np.ndarray, np.ndarray]:
    """u_accept [batch, n_nodes] and u_sample [batch], float32 in [0, 1)."""
    g = _rng(seed, 405)
    top = np.float32(1.0) - np.float32(2.0 ** -24)
    ua = np.minimum(g.random((batch, n_nodes), dtype=np.float32), top)
    us = np.minimum(g.random(batch, dtype=np.float32), top)
    return ua, us
