"""Pins for the oracle's forward passes.

* tree-masked cached pass == brute-force sequential causal forwards (paper Eq. 2 / Eq. 5:
  one parallel pass returns the k+1 next-token distributions);
* textbook causal forward == an independent forward assembled from torch library routines;
* structural invariants: cache split, non-ancestor independence, relabelling, chain == path.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import OracleWeights, causal_forward, verify_forward
from workloads import (ModelShape, WeightSource, gen_chain, gen_context_tokens, gen_draft_tokens,
                       gen_tree, tree_depths)
from helpers import MICRO, oracle_weights, path_to, prefill

VARIANTS = [
    MICRO,
    MICRO.with_(name="mha", n_q_heads=4, n_kv_heads=4),
    MICRO.with_(name="mqa", n_q_heads=4, n_kv_heads=1),
    MICRO.with_(name="wide_q", n_q_heads=6, n_kv_heads=2, head_dim=16),   # nq*d != hidden
    MICRO.with_(name="bf16", dtype="bf16"),
    MICRO.with_(name="three_layers", n_layers=3, rope_base=5e5),
    MICRO.with_(name="qk_norm", qk_norm=True, n_layers=3),
    MICRO.with_(name="qk_norm_bf16", qk_norm=True, dtype="bf16"),
]


def torch_causal_forward(shape, seed, tokens, positions):
    """Independent fp64 forward built from torch library routines (f32 storage mode)."""
    ws = WeightSource(shape, seed)
    t = lambda name, l=0: torch.from_numpy(ws.get(name, l).astype(np.float64))
    T = len(tokens)
    nq, nkv, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    x = F.embedding(torch.as_tensor(np.asarray(tokens), dtype=torch.long), t("embed"))
    inv = torch.tensor(shape.rope_base, dtype=torch.float64) ** (-torch.arange(0, d, 2, dtype=torch.float64) / d)
    ang = torch.as_tensor(np.asarray(positions), dtype=torch.float64)[:, None] * inv[None]
    rot = torch.polar(torch.ones_like(ang), ang)  # e^{i angle}, [T, d/2]

    def rope(u):  # [T, heads, d]; pairs (j, j+d/2) as complex numbers
        z = torch.complex(u[..., : d // 2], u[..., d // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    for l in range(shape.n_layers):
        h = F.rms_norm(x, (shape.hidden,), t("norm_attn", l), shape.rms_eps)
        q, k = F.linear(h, t("wq", l)).view(T, nq, d), F.linear(h, t("wk", l)).view(T, nkv, d)
        if shape.qk_norm:   # RMSNorm over the head dimension, before the rotary embedding
            q = F.rms_norm(q, (d,), t("q_norm", l), shape.rms_eps)
            k = F.rms_norm(k, (d,), t("k_norm", l), shape.rms_eps)
        q = rope(q).transpose(0, 1)   # [nq, T, d]
        k = rope(k).transpose(0, 1)
        v = F.linear(h, t("wv", l)).view(T, nkv, d).transpose(0, 1)
        k = k.repeat_interleave(nq // nkv, dim=0)
        v = v.repeat_interleave(nq // nkv, dim=0)
        o = F.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0]
        x = x + F.linear(o.transpose(0, 1).reshape(T, nq * d), t("wo", l))
        h = F.rms_norm(x, (shape.hidden,), t("norm_ffn", l), shape.rms_eps)
        x = x + F.linear(F.silu(F.linear(h, t("w_gate", l))) * F.linear(h, t("w_up", l)), t("w_down", l))
    h = F.rms_norm(x, (shape.hidden,), t("final_norm"), shape.rms_eps)
    return F.linear(h, t("lm_head")).numpy()


@pytest.mark.parametrize("shape", [v for v in VARIANTS if v.dtype == "f32"], ids=lambda s: s.name)
def test_causal_forward_equals_torch_library_forward(shape):
    seed = 11
    toks = gen_context_tokens(shape.vocab, 13, seed)
    pos = np.arange(13) + 5
    got = causal_forward(oracle_weights(shape, seed), shape, toks, positions=pos)["logits"]
    want = torch_causal_forward(shape, seed, toks, pos)
    assert np.max(np.abs(got - want)) < 1e-10


@pytest.mark.parametrize("shape", VARIANTS, ids=lambda s: s.name)
def test_tree_pass_equals_sequential_autoregressive_forwards(shape):
    seed, C, M = 5, 9, 11
    W = oracle_weights(shape, seed)
    ctx = gen_context_tokens(shape.vocab, C, seed)
    parents = gen_tree(M, 4, 3, seed)
    toks = gen_draft_tokens(parents, shape.vocab, seed)
    pos = C + tree_depths(parents)
    Kc, Vc = prefill(shape, seed, ctx)
    out = verify_forward(W, shape, Kc, Vc, toks, parents, pos)
    for i in range(M):
        seq = list(ctx) + [int(toks[j]) for j in path_to(parents, i)]
        ref = causal_forward(W, shape, seq, last_only=True, n_cached=C)
        assert np.max(np.abs(out["logits"][i] - ref["logits"][0])) < 1e-9, i
        # what the pass appends to the cache for node i is what a prefill would have stored
        assert np.max(np.abs(out["k_new"][:, :, i] - ref["K"][:, :, -1])) < 1e-10
        assert np.max(np.abs(out["v_new"][:, :, i] - ref["V"][:, :, -1])) < 1e-10


def test_cache_split_invariance():
    """(C=12, chain of 6) == (C=8, the last 4 context tokens as extra chain nodes) == (C=0, all nodes)."""
    shape, seed = MICRO, 3
    W = oracle_weights(shape, seed)
    ctx = gen_context_tokens(shape.vocab, 12, seed)
    chain = gen_draft_tokens(gen_chain(6), shape.vocab, seed)
    Kc, Vc = prefill(shape, seed, ctx)
    a = verify_forward(W, shape, Kc, Vc, chain, gen_chain(6), 12 + np.arange(6))["logits"]
    Kc8, Vc8 = prefill(shape, seed, ctx[:8])
    toks_b = np.concatenate([ctx[8:], chain])
    b = verify_forward(W, shape, Kc8, Vc8, toks_b, gen_chain(10), 8 + np.arange(10))["logits"]
    K0, V0 = prefill(shape, seed, ctx[:0])
    toks_c = np.concatenate([ctx, chain])
    c = verify_forward(W, shape, K0, V0, toks_c, gen_chain(18), np.arange(18))["logits"]
    assert np.max(np.abs(a - b[4:])) < 1e-10
    assert np.max(np.abs(a - c[12:])) < 1e-10


def test_non_ancestor_independence_and_relabelling():
    shape, seed, C, M = MICRO, 8, 6, 12
    W = oracle_weights(shape, seed)
    ctx = gen_context_tokens(shape.vocab, C, seed)
    Kc, Vc = prefill(shape, seed, ctx)
    parents = gen_tree(M, 4, 3, seed)
    toks = gen_draft_tokens(parents, shape.vocab, seed)
    pos = C + tree_depths(parents)
    base = verify_forward(W, shape, Kc, Vc, toks, parents, pos)["logits"]
    for j in range(1, M):
        t2 = toks.copy(); t2[j] = (t2[j] + 1) % shape.vocab
        out = verify_forward(W, shape, Kc, Vc, t2, parents, pos)["logits"]
        for i in range(M):
            if j in path_to(parents, i):
                assert not np.array_equal(out[i], base[i])
            else:
                assert np.array_equal(out[i], base[i]), (i, j)
    # another topological order permutes outputs only
    g = np.random.default_rng(0)
    keys = tree_depths(parents) + g.uniform(0, 0.9, M)  # random order within a level
    order = np.argsort(keys, kind="stable")
    new_id = np.empty(M, dtype=int); new_id[order] = np.arange(M)
    p2 = np.array([-1 if parents[o] < 0 else new_id[parents[o]] for o in order])
    out2 = verify_forward(W, shape, Kc, Vc, toks[order], p2, pos[order])["logits"]
    assert np.max(np.abs(out2 - base[order])) < 1e-12


def test_single_path_tree_equals_chain_and_position_shift():
    shape, seed, C = MICRO, 21, 7
    W = oracle_weights(shape, seed)
    ctx = gen_context_tokens(shape.vocab, C, seed)
    Kc, Vc = prefill(shape, seed, ctx)
    parents = gen_tree(9, 3, 3, seed)
    toks = gen_draft_tokens(parents, shape.vocab, seed)
    full = verify_forward(W, shape, Kc, Vc, toks, parents, C + tree_depths(parents))["logits"]
    leaf = 8
    p = path_to(parents, leaf)
    chain = verify_forward(W, shape, Kc, Vc, toks[p], gen_chain(len(p)), C + np.arange(len(p)))["logits"]
    assert np.max(np.abs(chain - full[p])) < 1e-10
    # rotary shift invariance: everything moved by +1000 positions, cache re-prefilled there
    Ks, Vs = prefill(shape, seed, ctx, start_pos=1000)
    sh = verify_forward(W, shape, Ks, Vs, toks, parents, 1000 + C + tree_depths(parents))["logits"]
    assert np.max(np.abs(sh - full)) < 1e-8


def test_final_hidden_is_what_the_lm_head_maps_to_the_logits():
    """The exported feature is pinned through the logits (themselves pinned above): the vocabulary is
    larger than the hidden size, so a least-squares solve of lm_head . h = logits (numpy's LAPACK
    routine) has one solution, which must be final_hidden."""
    from oracle import OracleWeights, verify_forward
    from workloads import SHAPES, WeightSource, gen_draft_tokens, gen_tree, tree_depths
    shape, seed = SHAPES["tiny"], 3
    W = OracleWeights(WeightSource(shape, seed).get)
    parents = gen_tree(12, 4, 3, seed)
    d = shape.head_dim
    rng = np.random.default_rng(0)
    k = rng.standard_normal((shape.n_layers, shape.n_kv_heads, 20, d))
    v = rng.standard_normal((shape.n_layers, shape.n_kv_heads, 20, d))
    out = verify_forward(W, shape, k, v, gen_draft_tokens(parents, shape.vocab, seed), parents, 20 + tree_depths(parents))
    head = np.asarray(W("lm_head"), dtype=np.float64)
    assert head.shape[0] > head.shape[1]
    sol, _, rank, _ = np.linalg.lstsq(head, out["logits"].T, rcond=None)
    assert rank == shape.hidden
    assert np.allclose(sol.T, out["final_hidden"], rtol=0, atol=1e-9)


# ---- the cache boundary in bf16 storage: the two readings of "what does a node see of the
# other nodes of its own pass", each pinned on its own, and the distance between them bounded

def torch_causal_forward_rounded_kv(shape, seed, tokens, positions):
    """The torch-library forward with a bf16 KV cache that is written before it is read: keys
    (after the rotary embedding) and values pass through torch's own bfloat16 type on their way
    into attention; everything else stays fp64."""
    ws = WeightSource(shape, seed)
    t = lambda name, l=0: torch.from_numpy(ws.get(name, l).astype(np.float64))
    T = len(tokens)
    nq, nkv, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    cached = lambda u: u.to(torch.bfloat16).to(torch.float64)
    x = F.embedding(torch.as_tensor(np.asarray(tokens), dtype=torch.long), t("embed"))
    inv = torch.tensor(shape.rope_base, dtype=torch.float64) ** (-torch.arange(0, d, 2, dtype=torch.float64) / d)
    ang = torch.as_tensor(np.asarray(positions), dtype=torch.float64)[:, None] * inv[None]
    rot = torch.polar(torch.ones_like(ang), ang)

    def rope(u):
        z = torch.complex(u[..., : d // 2], u[..., d // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    for l in range(shape.n_layers):
        h = F.rms_norm(x, (shape.hidden,), t("norm_attn", l), shape.rms_eps)
        q = rope(F.linear(h, t("wq", l)).view(T, nq, d)).transpose(0, 1)
        k = cached(rope(F.linear(h, t("wk", l)).view(T, nkv, d))).transpose(0, 1)
        v = cached(F.linear(h, t("wv", l)).view(T, nkv, d)).transpose(0, 1)
        k = k.repeat_interleave(nq // nkv, dim=0)
        v = v.repeat_interleave(nq // nkv, dim=0)
        o = F.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0]
        x = x + F.linear(o.transpose(0, 1).reshape(T, nq * d), t("wo", l))
        h = F.rms_norm(x, (shape.hidden,), t("norm_ffn", l), shape.rms_eps)
        x = x + F.linear(F.silu(F.linear(h, t("w_gate", l))) * F.linear(h, t("w_up", l)), t("w_down", l))
    h = F.rms_norm(x, (shape.hidden,), t("final_norm"), shape.rms_eps)
    return F.linear(h, t("lm_head")).numpy()


BF16_VARIANTS = [MICRO.with_(name="bf16", dtype="bf16"),
                 MICRO.with_(name="bf16_mqa_3l", dtype="bf16", n_layers=3, n_q_heads=4, n_kv_heads=1)]


@pytest.mark.parametrize("shape", BF16_VARIANTS, ids=lambda s: s.name)
def test_bf16_cache_forward_equals_torch_library_forward_with_rounded_kv(shape):
    """Reading "stored" needs no cache boundary: it is the plain causal forward of a model whose
    keys and values live in bf16.  Pinned against torch's rounding and torch's attention."""
    seed = 12
    toks = gen_context_tokens(shape.vocab, 14, seed)
    pos = np.arange(14) + 3
    got = causal_forward(oracle_weights(shape, seed), shape, toks, positions=pos, in_pass_kv="stored")["logits"]
    want = torch_causal_forward_rounded_kv(shape, seed, toks, pos)
    assert np.max(np.abs(got - want)) < 1e-10
    plain = causal_forward(oracle_weights(shape, seed), shape, toks, positions=pos)["logits"]
    assert np.max(np.abs(got - plain)) > 1e-6          # the rounding is really there


@pytest.mark.parametrize("shape", BF16_VARIANTS, ids=lambda s: s.name)
def test_tree_pass_equals_sequential_decoding_through_a_bf16_cache(shape):
    """Under reading "stored" the tree pass equals brute-force sequential forwards with no cache
    boundary argument at all: every key and value is the stored one on both sides."""
    seed, C, M = 6, 9, 11
    W = oracle_weights(shape, seed)
    ctx = gen_context_tokens(shape.vocab, C, seed)
    parents = gen_tree(M, 4, 3, seed)
    toks = gen_draft_tokens(parents, shape.vocab, seed)
    pos = C + tree_depths(parents)
    pre = causal_forward(W, shape, ctx, last_only=True, in_pass_kv="stored")   # the cache of a decoder of this reading
    out = verify_forward(W, shape, pre["K"], pre["V"], toks, parents, pos, in_pass_kv="stored")
    for i in range(M):
        seq = list(ctx) + [int(toks[j]) for j in path_to(parents, i)]
        ref = causal_forward(W, shape, seq, last_only=True, in_pass_kv="stored")
        assert np.max(np.abs(out["logits"][i] - ref["logits"][0])) < 1e-9, i


def test_the_two_cache_boundary_readings_differ_by_less_than_the_tie_tolerances():
    """The draft nodes of a pass see each other's keys / values unrounded; the other reading
    rounds them as the cache would.  Measured here on the bf16 test model: logits move by <= 1e-2 absolute (about 2e-4 of their magnitude, a
    hundredth of the 2e-2 bf16 bar), the routing statistics by <= 3e-3, and no decision changes
    unless a node of the walk sits that close to the threshold or to a top-2 tie."""
    from oracle import CRIT_MARGIN, CRIT_TOP1, decide, node_stats
    from workloads import SHAPES
    shape = SHAPES["tiny_bf16"]
    worst = np.zeros(3)
    compared = 0
    for seed in range(2):
        W = oracle_weights(shape, seed)
        C, M = 96, 40
        ctx = gen_context_tokens(shape.vocab, C, seed)
        K, V = prefill(shape, seed, ctx)
        par = gen_tree(M, 8, 4, seed)
        tok = gen_draft_tokens(par, shape.vocab, seed)
        pos = C + tree_depths(par)
        a = verify_forward(W, shape, K, V, tok, par, pos)["logits"]
        b = verify_forward(W, shape, K, V, tok, par, pos, in_pass_kv="stored")["logits"]
        sa, sb = node_stats(a), node_stats(b)
        worst = np.maximum(worst, [np.abs(a - b).max(), np.abs(a - b).max() / np.abs(a).max(),
                                   max(np.abs(sa["conf"] - sb["conf"]).max(), np.abs(sa["margin"] - sb["margin"]).max())])
        clear = (sa["l1"] - sa["l2"]) >= 2e-2
        assert np.array_equal(sa["argmax"][clear], sb["argmax"][clear])
        for crit in (CRIT_MARGIN, CRIT_TOP1):
            stat = sa["margin"] if crit == CRIT_MARGIN else sa["conf"]
            for lam in (0.0, 0.1, 0.3, 0.5, 0.7, 0.9):
                da = decide(tok, par, sa["argmax"], sa["conf"], sa["margin"], lam, crit, 1)
                db = decide(tok, par, sb["argmax"], sb["conf"], sb["margin"], lam, crit, 1)
                touched = sorted(set(da["path"]) | set(db["path"]))
                near = any(abs(stat[i] - lam) < 3e-3 or not clear[i] for i in touched)
                if not near:
                    compared += 1
                    assert (da["accepted_len"], da["token"], da["escalate"]) == (db["accepted_len"], db["token"], db["escalate"])
    print("max |dlogit| %.3g (relative %.3g), max |dstat| %.3g" % tuple(worst))
    assert worst[0] <= 1e-2 and worst[1] <= 5e-4 and worst[2] <= 3e-3
    assert worst[0] >= 1e-4          # the readings do differ: the bound is not vacuous
    assert compared >= 12


def test_per_layer_hidden_states_and_the_adapter():
    """hidden[l] (the residual stream after layer l, what a multi-layer drafter is fed) is pinned by
    consistency with passes that are themselves pinned: it is the last hidden state of the same model
    cut to l + 1 layers, and its final RMSNorm is final_hidden.  The adapter is one affine map:
    identity weights return the features plus the bias, and it is linear."""
    from oracle import adapter, rmsnorm
    shape, seed, C, M = MICRO.with_(n_layers=3), 8, 7, 9
    W = oracle_weights(shape, seed)
    ctx = gen_context_tokens(shape.vocab, C, seed)
    parents = gen_tree(M, 4, 3, seed)
    toks = gen_draft_tokens(parents, shape.vocab, seed)
    pos = C + tree_depths(parents)
    Kc, Vc = prefill(shape, seed, ctx)
    full = verify_forward(W, shape, Kc, Vc, toks, parents, pos, keep_hidden=True)
    assert full["hidden"].shape == (3, M, shape.hidden)
    for l in range(3):
        cut = verify_forward(W, shape.with_(n_layers=l + 1), Kc[: l + 1], Vc[: l + 1], toks, parents, pos, keep_hidden=True)
        assert np.array_equal(cut["hidden"][l], full["hidden"][l])
    assert np.allclose(rmsnorm(full["hidden"][2], W("final_norm"), shape.rms_eps), full["final_hidden"], rtol=0, atol=1e-12)
    assert np.abs(full["hidden"][0] - full["hidden"][2]).max() > 1e-3
    f = full["final_hidden"]
    rng = np.random.default_rng(1)
    b = rng.standard_normal(shape.hidden)
    assert np.allclose(adapter(f, np.eye(shape.hidden), b), f + b, rtol=0, atol=1e-14)
    A = rng.standard_normal((20, shape.hidden))
    want = np.array([[sum(A[o, i] * f[r, i] for i in range(shape.hidden)) for o in range(20)] for r in range(M)])
    assert np.allclose(adapter(f, A), want, rtol=0, atol=1e-12)
    b20 = rng.standard_normal(20)
    assert np.allclose(adapter(2 * f, A, b20), 2 * adapter(f, A) + b20, rtol=0, atol=1e-12)
