"""GPU: committing a verified path (trispec_kv_commit) and several rounds of
draft -> verify -> commit through the C ABI, against the oracle's rounds (Sec. 2.1, Alg. 1)."""
import numpy as np
import pytest
import torch

from oracle import CRIT_MARGIN, greedy_decode, tie_flags, verify_rounds
from paper_2601_23180_amd import KVCache, Verifier
from workloads import SHAPES, gen_chain, gen_context_tokens, gen_draft_tokens, gen_tree, tree_depths

from gpu_helpers import capacity_for, device_model
from helpers import oracle_weights, prefill

pytestmark = pytest.mark.gpu


def mixed_drafts(W, shape, seed, n_nodes):
    """Seeded trees; along the path to the deepest leaf the first r drafts are the oracle's own
    greedy continuation (r varies per round), so accepted lengths cover 0 .. depth."""
    def fn(r, seq):
        parents = gen_tree(n_nodes, 5, 3, seed + r)
        tokens = gen_draft_tokens(parents, shape.vocab, seed + 17 * r)
        depth = tree_depths(parents)
        leaf = int(np.argmax(depth))
        path = [leaf]
        while parents[path[-1]] >= 0:
            path.append(int(parents[path[-1]]))
        path = path[::-1]
        n_right = (r * 2) % len(path)
        cont = greedy_decode(W, shape, seq, n_right)[len(seq):]
        for node, tok in zip(path[1:], cont):
            tokens[node] = tok
            # keep siblings distinct
            for s in np.nonzero(parents == parents[node])[0]:
                if s != node and tokens[s] == tok:
                    tokens[s] = (tok + 1) % shape.vocab
        return parents, tokens
    return fn


def gpu_rounds(shape, seed, prompt, draft_fn, n_rounds, n_nodes):
    model = device_model(shape, seed)
    K, V = prefill(shape, seed, prompt[:-1])
    C0 = len(prompt) - 1
    kv = KVCache(model, 1, capacity_for(C0 + n_rounds * n_nodes + n_nodes))
    kv.k.fill_(float("nan")); kv.v.fill_(float("nan"))
    kv.k[:, 0, :, :C0, :] = torch.from_numpy(np.asarray(K, dtype=np.float32)).cuda().to(kv.k.dtype)
    kv.v[:, 0, :, :, :C0] = torch.from_numpy(np.asarray(V, dtype=np.float32)).cuda().to(kv.v.dtype).transpose(-1, -2)
    kv.set_len([C0])
    ver = Verifier(model, 1, n_nodes)
    seq = [int(t) for t in prompt]
    rounds = []
    for r in range(n_rounds):
        parents, tokens = draft_fn(r, seq)
        tokens = np.asarray(tokens, dtype=np.int32).copy()
        tokens[0] = seq[-1]
        C = kv.ctx_len[0]
        pos = (C + tree_depths(parents)).astype(np.int32)
        out = ver.verify(kv, torch.from_numpy(tokens[None]).cuda(), parents[None], torch.from_numpy(pos[None]).cuda(),
                         0.0, CRIT_MARGIN, 1, want_logits=False)
        torch.cuda.synchronize()
        path = [int(v) for v in out["path"][0].cpu().numpy() if v >= 0]
        rounds.append({"ctx_len": C, "accepted_len": int(out["accepted_len"][0]), "token": int(out["token"][0]),
                       "escalate": int(out["escalate"][0]), "path": path})
        kv.commit([path])
        seq += [int(tokens[i]) for i in path[1:]] + [int(out["token"][0])]
    torch.cuda.synchronize()
    return seq, rounds, kv


def until_compared_in_full(run, seeds):
    """A tie inside the tolerance may change a round, and then every round after it: such a run is
    excused (its excuse is asserted inside `run`, which returns False) and COUNTED, and the next
    seed is taken, until one run compares in full.  Returns the number of excused runs."""
    for n, seed in enumerate(seeds):
        if run(seed):
            return n
    pytest.fail(f"all {len(seeds)} seeds were changed by a tie: nothing was compared in full")


@pytest.mark.parametrize("shape_name,seed", [("tiny", 3), ("tiny_bf16", 4)])
def test_rounds_match_the_oracle_and_greedy_decoding(shape_name, seed):
    assert until_compared_in_full(lambda s: _rounds_vs_oracle(shape_name, s), [seed, seed + 50, seed + 100]) <= 1


def _rounds_vs_oracle(shape_name, seed):
    shape, n_nodes, n_rounds = SHAPES[shape_name], 12, 5
    W = oracle_weights(shape, seed)
    prompt = gen_context_tokens(shape.vocab, 20, seed).tolist()
    fn = mixed_drafts(W, shape, seed, n_nodes)
    want = verify_rounds(W, shape, prompt, fn, n_rounds)
    seq, rounds, kv = gpu_rounds(shape, seed, prompt, fn, n_rounds, n_nodes)
    # a tie inside 1e-3 on a node the walk touches may change a round (and everything after it)
    for r, (g, w) in enumerate(zip(rounds, want["rounds"])):
        d = w["decision"]
        same = (g["accepted_len"] == d["accepted_len"] and g["token"] == d["token"] and g["path"] == [int(v) for v in d["path"]])
        if not same:
            flags = tie_flags(w["stats"], 0.0, CRIT_MARGIN)
            assert any(flags[i] for i in set(g["path"]) | set(int(v) for v in d["path"])), (r, g, d)
            return False
        assert g["ctx_len"] == w["ctx_len"] and g["escalate"] == 0
    assert seq == want["sequence"]
    assert max(g["accepted_len"] for g in rounds) >= 3            # the planted prefixes were accepted and committed
    if shape.dtype == "f32":
        assert seq == greedy_decode(W, shape, prompt, len(seq) - len(prompt))
    # the committed cache is the oracle's committed cache (bf16: half an ulp where a value sits on a boundary)
    Cn = kv.ctx_len[0]
    assert Cn == want["k_ctx"].shape[2]
    kg = kv.k[:, 0, :, :Cn, :].float().cpu().numpy()
    vg = kv.v[:, 0, :, :, :Cn].float().cpu().numpy().transpose(0, 1, 3, 2)
    tol = (lambda w: 1e-4) if shape.dtype == "f32" else (lambda w: np.abs(w) * 2 ** -7 + 1e-4)
    assert np.all(np.abs(kg - want["k_ctx"]) <= tol(want["k_ctx"]))
    assert np.all(np.abs(vg - want["v_ctx"]) <= tol(want["v_ctx"]))
    return True


def test_commit_moves_exactly_the_path_rows():
    shape, seed, n_nodes = SHAPES["tiny_bf16"], 9, 20
    model = device_model(shape, seed)
    kv = KVCache(model, 2, 128)
    g = torch.Generator(device="cuda").manual_seed(1)
    kv.k.copy_(torch.randn(kv.k.shape, device="cuda", generator=g).to(kv.k.dtype))
    kv.v.copy_(torch.randn(kv.v.shape, device="cuda", generator=g).to(kv.v.dtype))
    k0, v0 = kv.k.clone(), kv.v.clone()
    kv.set_len([40, 17])
    paths = [[0, 3, 4, 11, 19], [2]]
    kv.commit(paths)
    torch.cuda.synchronize()
    assert kv.ctx_len == [45, 18]
    for b, (C, p) in enumerate(zip([40, 17], paths)):
        for i, n in enumerate(p):
            assert torch.equal(kv.k[:, b, :, C + i, :], k0[:, b, :, C + n, :])
            assert torch.equal(kv.v[:, b, :, :, C + i], v0[:, b, :, :, C + n])
        untouched = [s for s in range(128) if not (C <= s < C + len(p))]
        assert torch.equal(kv.k[:, b, :, untouched, :], k0[:, b, :, untouched, :])
        assert torch.equal(kv.v[:, b, :, :, untouched], v0[:, b, :, :, untouched])


# ---- the ternary scheme with two models (Alg. 1) through the product's round driver

def _run_decoder(shape, seed_p, seed_t, prompt, drafts, n_rounds, lam, max_nodes=64):
    from paper_2601_23180_amd import TernaryDecoder
    dec = TernaryDecoder(device_model(shape, seed_p), device_model(shape, seed_t), 256, max_nodes=max_nodes)
    dec.start(prompt)
    recs = [dec.round(*drafts(r, dec.seq), lam) for r in range(n_rounds)]
    return dec, recs


def test_taking_over_a_sequence_continues_it_exactly():
    """trispec_ternary_resume: a driver that is handed the emitted sequence again (as after rounds the
    caller ran by other means) goes on exactly like one that never lost it."""
    shape = SHAPES["tiny"]
    Wp = oracle_weights(shape, 51)
    prompt = gen_context_tokens(shape.vocab, 10, 51).tolist()
    drafts = mixed_drafts(Wp, shape, 51, 12)
    a, recs_a = _run_decoder(shape, 51, 52, prompt, drafts, 6, 0.35)
    from paper_2601_23180_amd import TernaryDecoder
    b = TernaryDecoder(device_model(shape, 51), device_model(shape, 52), 256)
    b.start(prompt)
    recs_b = []
    for r in range(6):
        b._stale = True                      # forces the take-over path before every round
        recs_b.append(b.round(*drafts(r, b.seq), 0.35))
    assert recs_a == recs_b and a.seq == b.seq
    assert a.kv_p.ctx_len == b.kv_p.ctx_len and a.kv_t.ctx_len == b.kv_t.ctx_len
    assert any(r["escalate"] for r in recs_a) and not all(r["escalate"] for r in recs_a)


@pytest.mark.parametrize("shape_name,lam,max_nodes", [("tiny", 0.0, 64), ("tiny", 0.35, 64), ("tiny", 2.0, 64),
                                                       ("tiny", 0.35, 16), ("tiny_bf16", 0.35, 64)])
def test_ternary_rounds_match_the_oracle(shape_name, lam, max_nodes):
    run = lambda s: _ternary_rounds_vs_oracle(shape_name, lam, max_nodes, s, s + 1)
    assert until_compared_in_full(run, [41, 141, 241]) <= 1


def _ternary_rounds_vs_oracle(shape_name, lam, max_nodes, seed_p, seed_t):
    from oracle import trispec_rounds
    shape, n_rounds = SHAPES[shape_name], 8
    Wp, Wt = oracle_weights(shape, seed_p), oracle_weights(shape, seed_t)
    prompt = gen_context_tokens(shape.vocab, 12, seed_p).tolist()
    drafts = mixed_drafts(Wt if lam > 1 else Wp, shape, seed_p, 12)
    want = trispec_rounds(Wp, shape, Wt, shape, prompt, drafts, n_rounds, lam, max_nodes=max_nodes)
    dec, recs = _run_decoder(shape, seed_p, seed_t, prompt, drafts, n_rounds, lam, max_nodes)
    for r, (g, w) in enumerate(zip(recs, want["rounds"])):
        ok = g["escalate"] == w["escalate"] and g["proxy"]["path"] == [int(v) for v in w["proxy"]["path"]]
        if ok and g["escalate"]:
            ok = (g["target"]["path"] == [int(v) for v in w["target"]["path"]] and g["target"]["token"] == w["target"]["token"]
                  and g["n_forced_t"] == w["n_forced_t"] and g["catch_up"] == w["catch_up"])
        elif ok:
            ok = g["proxy"]["token"] == w["proxy"]["token"]
        if not ok:     # only a tie inside the tolerance may change a round
            flags = tie_flags(w["proxy_stats"], lam, CRIT_MARGIN)
            tflags = tie_flags(w["target_stats"], 0.0, CRIT_MARGIN) if w["escalate"] else []
            assert any(flags) or any(tflags), (r, g, w["proxy"], w.get("target"))
            return False
    assert dec.seq == want["sequence"]
    n_esc = sum(g["escalate"] for g in recs)
    assert dec.target_passes == n_esc
    if lam == 0.0:
        assert n_esc == 0
    if lam > 1:
        assert n_esc == n_rounds
        if shape.dtype == "f32":      # lossless with respect to the target
            assert dec.seq == greedy_decode(Wt, shape, prompt, len(dec.seq) - len(prompt))
    if lam == 0.0 and shape.dtype == "f32":
        assert dec.seq == greedy_decode(Wp, shape, prompt, len(dec.seq) - len(prompt))
    if max_nodes == 16:
        assert any(g["catch_up"] for g in recs) or any(g["escalate"] and g["n_forced_t"] > len(g["proxy"]["path"]) for g in recs)
    # both caches cover the emitted sequence up to where each model has seen it
    assert dec.kv_p.ctx_len[0] == len(dec.seq) - 1 == want["kp"].shape[2]
    assert dec.kv_t.ctx_len[0] == want["kt"].shape[2]
    tol = (lambda w: 2e-4) if shape.dtype == "f32" else (lambda w: np.abs(w) * 2 ** -7 + 2e-4)
    for kv, kw, vw in ((dec.kv_p, want["kp"], want["vp"]), (dec.kv_t, want["kt"], want["vt"])):
        n = kw.shape[2]
        kg = kv.k[:, 0, :, :n, :].float().cpu().numpy()
        vg = kv.v[:, 0, :, :, :n].float().cpu().numpy().transpose(0, 1, 3, 2)
        assert np.all(np.abs(kg - kw) <= tol(kw)) and np.all(np.abs(vg - vw) <= tol(vw))
    return True


# ---- rounds at temperature > 0 on draft chains (Alg. 1 as printed)

def _model_drafter(Wd, shape, k, temperature, seed, noise):
    """Drafts sampled autoregressively from softmax((oracle logits of Wd + noise) / T) with numpy's
    generator; the same recorded inputs then go to the GPU driver."""
    from oracle import causal_forward, tempered_softmax

    def fn(r, seq, _cache_len):
        rng = np.random.default_rng(seed * 1000 + r)
        cur, toks, rows = list(seq), [0], []
        for _ in range(k):
            lg = causal_forward(Wd, shape, cur, last_only=True, n_cached=len(cur) - 1)["logits"][0]
            q = tempered_softmax(lg + noise * rng.standard_normal(lg.shape), temperature).astype(np.float32)
            c = np.cumsum(q.astype(np.float64))
            x = min(int(np.searchsorted(c, rng.random() * c[-1], side="right")), len(q) - 1)
            toks.append(x); rows.append(q); cur.append(x)
        top = np.float32(1.0) - np.float32(2.0 ** -24)
        u = lambda n: np.minimum(rng.random(n, dtype=np.float32), top)
        return {"tokens": np.array(toks, dtype=np.int32), "p_draft": np.stack(rows),
                "u_accept_p": u(k + 1), "u_sample_p": float(u(1)[0]), "u_accept_t": u(k + 1), "u_sample_t": float(u(1)[0])}
    return fn


@pytest.mark.parametrize("shape_name,lam,max_nodes", [("tiny", 0.0, 64), ("tiny", 0.25, 64), ("tiny", 2.0, 64),
                                                       ("tiny", 0.25, 12), ("tiny_bf16", 0.25, 64)])
def test_sampling_rounds_match_the_oracle(shape_name, lam, max_nodes):
    run = lambda s: _sampling_rounds_vs_oracle(shape_name, lam, max_nodes, s, s + 1)
    assert until_compared_in_full(run, [41, 141, 241]) <= 1


def _sampling_rounds_vs_oracle(shape_name, lam, max_nodes, seed_p, seed_t):
    from oracle import trispec_sample_rounds
    from paper_2601_23180_amd import TernaryDecoder
    shape, n_rounds, T, k = SHAPES[shape_name], 8, 0.8, 4
    Wp, Wt = oracle_weights(shape, seed_p), oracle_weights(shape, seed_t)
    prompt = gen_context_tokens(shape.vocab, 12, seed_p).tolist()
    log = {}
    drafter = _model_drafter(Wp, shape, k, T, seed_p, noise=0.6)

    def recording(r, seq, c):
        log[r] = drafter(r, seq, c)
        return log[r]
    want = trispec_sample_rounds(Wp, shape, Wt, shape, prompt, recording, n_rounds, lam, T, max_nodes=max_nodes)
    dec = TernaryDecoder(device_model(shape, seed_p), device_model(shape, seed_t), 256, max_nodes=max_nodes)
    dec.start(prompt)
    tol = 3e-4 if shape.dtype == "f32" else 5e-3
    for r in range(n_rounds):
        d, w = log[r], want["rounds"][r]
        g = dec.round_sample(d["tokens"], d["p_draft"], d["u_accept_p"], d["u_sample_p"], d["u_accept_t"],
                             d["u_sample_t"], lam, T)
        ok = g["escalate"] == w["escalate"] and g["proxy"]["path"] == list(w["proxy"]["path"])
        if ok and g["escalate"]:
            ok = (g["target"]["path"] == list(w["target"]["path"]) and g["target"]["token"] == w["target"]["token"]
                  and g["n_forced_t"] == w["n_forced_t"] and g["catch_up"] == w["catch_up"])
        elif ok:
            ok = g["proxy"]["token"] == w["proxy"]["token"]
        if not ok:   # only a comparison within rounding of its boundary may change a round
            close = w["proxy"]["slack"] < tol or (w["escalate"] and w["target"]["slack"] < tol)
            for side in ("proxy", "target"):
                o = w.get(side)
                if o is not None and o["mass"] is not None:
                    c = np.cumsum(o["mass"])
                    us = d["u_sample_p"] if side == "proxy" else d["u_sample_t"]
                    pos = np.searchsorted(c, us * c[-1], side="right")
                    edges = c[max(pos - 1, 0): pos + 1]
                    close = close or bool(np.any(np.abs(edges - us * c[-1]) < tol))
            assert close, (r, g, w["proxy"]["path"], w.get("target", {}).get("path"))
            return False
    assert dec.seq == want["sequence"]
    n_esc = sum(w["escalate"] for w in want["rounds"])
    assert dec.target_passes == n_esc
    assert (lam == 0.0 and n_esc == 0) or (lam > 1 and n_esc == n_rounds) or 0 < n_esc < n_rounds
    assert dec.kv_p.ctx_len[0] == len(dec.seq) - 1 == want["kp"].shape[2]
    assert dec.kv_t.ctx_len[0] == want["kt"].shape[2]
    if max_nodes == 12:
        assert any(w["catch_up"] for w in want["rounds"]) or any(w["escalate"] and w["u"] > 0 for w in want["rounds"])
    return True


def test_sampling_rounds_after_a_long_lag_with_the_default_node_limit():
    """With the library's largest pass (128 nodes) the target may lag by more tokens than a sampling
    chain can hold (64 nodes): the driver must then take the lagging tokens in by plain passes first,
    and end where a driver limited to 64-node passes ends."""
    from paper_2601_23180_amd import TernaryDecoder
    shape, T, k = SHAPES["tiny"], 0.8, 4
    Wp = oracle_weights(shape, 71)
    prompt = gen_context_tokens(shape.vocab, 12, 71).tolist()
    drafter = _model_drafter(Wp, shape, k, T, 71, noise=0.6)
    runs = []
    for max_nodes in (128, 64):
        dec = TernaryDecoder(device_model(shape, 71), device_model(shape, 72), 512, max_nodes=max_nodes)
        dec.start(prompt)
        recs = []
        for r in range(34):
            lam = 0.0 if r < 32 else 2.0              # 32 rounds that end at the proxy, then two escalations
            d = drafter(r, dec.seq, dec.kv_p.ctx_len[0])
            recs.append(dec.round_sample(d["tokens"], d["p_draft"], d["u_accept_p"], d["u_sample_p"], d["u_accept_t"],
                                         d["u_sample_t"], lam, T))
        lag = len(dec.seq) - len(prompt)
        runs.append((dec.seq, dec.kv_p.ctx_len, dec.kv_t.ctx_len, [r["escalate"] for r in recs], recs[32]["catch_up"]))
        dec.close()
        assert lag > 64
    assert runs[0][:4] == runs[1][:4]
    assert runs[0][3][:32] == [0] * 32 and runs[0][3][32:] == [1, 1]
    assert runs[0][4] >= 1 and runs[1][4] >= 1        # both had to catch up before the escalated round
