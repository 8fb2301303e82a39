"""Pins of the oracle's commit / multi-round loop (Sec. 2.1, Alg. 1): with one verifier and
lambda = 0, rounds of draft -> verify -> commit emit exactly the tokens of plain greedy
autoregressive decoding, whatever the drafts are, and the committed cache is the textbook cache
of the emitted sequence."""
import numpy as np
import pytest

from oracle import causal_forward, commit, greedy_decode, verify_rounds
from workloads import gen_chain, gen_context_tokens, gen_draft_tokens, gen_tree

from helpers import MICRO, oracle_weights


def random_tree_drafts(shape, seed, n_nodes):
    def fn(r, seq):
        parents = gen_tree(n_nodes, 4, 3, seed + r)
        return parents, gen_draft_tokens(parents, shape.vocab, seed + 31 * r)
    return fn


def oracle_chain_drafts(W, shape, k, wrong_after=None):
    """Drafts = the verifier's own greedy continuation (a chain of k), optionally corrupted from
    draft position `wrong_after` on."""
    def fn(r, seq):
        cont = greedy_decode(W, shape, seq, k)[len(seq):]
        toks = np.array([0] + cont, dtype=np.int32)
        if wrong_after is not None:
            for j in range(wrong_after + 1, k + 1):
                toks[j] = (toks[j] + 1 + r) % shape.vocab
        return gen_chain(k + 1), toks
    return fn


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_random_drafts_emit_the_greedy_sequence(seed):
    shape = MICRO
    W = oracle_weights(shape, seed)
    prompt = gen_context_tokens(shape.vocab, 7, seed).tolist()
    res = verify_rounds(W, shape, prompt, random_tree_drafts(shape, seed, 9), n_rounds=5)
    n_new = len(res["sequence"]) - len(prompt)
    assert n_new >= 5
    assert res["sequence"] == greedy_decode(W, shape, prompt, n_new)


@pytest.mark.parametrize("wrong_after", [None, 0, 2])
def test_planted_chains_accept_what_is_right_and_commit_it(wrong_after):
    shape, seed, k = MICRO, 5, 4
    W = oracle_weights(shape, seed)
    prompt = gen_context_tokens(shape.vocab, 6, seed).tolist()
    res = verify_rounds(W, shape, prompt, oracle_chain_drafts(W, shape, k, wrong_after), n_rounds=3)
    want_len = k if wrong_after is None else wrong_after
    for rd in res["rounds"]:
        assert rd["decision"]["accepted_len"] == want_len and rd["decision"]["escalate"] == 0
    seq = res["sequence"]
    assert len(seq) == len(prompt) + 3 * (want_len + 1)
    assert seq == greedy_decode(W, shape, prompt, len(seq) - len(prompt))
    # the committed cache is the textbook cache of everything but the last emitted token
    ref = causal_forward(W, shape, seq[:-1])
    assert res["k_ctx"].shape == ref["K"].shape
    assert np.max(np.abs(res["k_ctx"] - ref["K"])) < 1e-9 and np.max(np.abs(res["v_ctx"] - ref["V"])) < 1e-9


def test_commit_is_a_gather_of_the_path_rows():
    rng = np.random.default_rng(0)
    k_ctx, v_ctx = rng.normal(size=(2, 2, 5, 8)), rng.normal(size=(2, 2, 5, 8))
    k_new, v_new = rng.normal(size=(2, 2, 9, 8)), rng.normal(size=(2, 2, 9, 8))
    k, v = commit(k_ctx, v_ctx, k_new, v_new, [0, 2, 7])
    assert k.shape == (2, 2, 8, 8)
    for l in range(2):
        for h in range(2):
            for i, n in enumerate([0, 2, 7]):
                assert np.array_equal(k[l, h, 5 + i], k_new[l, h, n]) and np.array_equal(v[l, h, 5 + i], v_new[l, h, n])
            assert np.array_equal(k[l, h, :5], k_ctx[l, h]) and np.array_equal(v[l, h, :5], v_ctx[l, h])


# ---- the ternary scheme (Alg. 1) with two models

def _two_models(seed_p, seed_t):
    return oracle_weights(MICRO, seed_p), oracle_weights(MICRO, seed_t)


def _mixed_drafts(Wref, shape, seed, n_nodes):
    """Seeded trees whose path to the deepest leaf starts with r tokens of Wref's greedy continuation."""
    from workloads import tree_depths

    def fn(r, seq):
        parents = gen_tree(n_nodes, 5, 3, seed + r)
        tokens = gen_draft_tokens(parents, shape.vocab, seed + 13 * r)
        leaf = int(np.argmax(tree_depths(parents)))
        path = [leaf]
        while parents[path[-1]] >= 0:
            path.append(int(parents[path[-1]]))
        path = path[::-1]
        cont = greedy_decode(Wref, shape, seq, (2 * r + 1) % len(path))[len(seq):]
        for node, tok in zip(path[1:], cont):
            tokens[node] = tok
            for s in np.nonzero(parents == parents[node])[0]:
                if s != node and tokens[s] == tok:
                    tokens[s] = (tok + 1) % shape.vocab
        return parents, tokens
    return fn


@pytest.mark.parametrize("lam", [0.0, 0.3, 2.0])
def test_same_model_as_proxy_and_target_is_greedy_decoding_at_any_threshold(lam):
    from oracle import trispec_rounds
    W = oracle_weights(MICRO, 11)
    prompt = gen_context_tokens(MICRO.vocab, 6, 11).tolist()
    res = trispec_rounds(W, MICRO, W, MICRO, prompt, _mixed_drafts(W, MICRO, 11, 10), 6, lam)
    seq = res["sequence"]
    assert seq == greedy_decode(W, MICRO, prompt, len(seq) - len(prompt))
    n_esc = sum(r["escalate"] for r in res["rounds"])
    assert (lam == 0.0 and n_esc == 0) or (lam == 2.0 and n_esc == 6) or lam == 0.3


def test_never_trusted_proxy_gives_the_targets_sequence_and_always_trusted_the_proxys():
    from oracle import trispec_rounds
    Wp, Wt = _two_models(21, 22)
    prompt = gen_context_tokens(MICRO.vocab, 6, 21).tolist()
    drafts = _mixed_drafts(Wt, MICRO, 21, 10)
    lossless = trispec_rounds(Wp, MICRO, Wt, MICRO, prompt, drafts, 6, 2.0)        # margin <= 1 < lambda
    seq = lossless["sequence"]
    assert seq == greedy_decode(Wt, MICRO, prompt, len(seq) - len(prompt))
    assert all(r["escalate"] for r in lossless["rounds"])
    assert max(r["target"]["accepted_len"] for r in lossless["rounds"]) >= 2        # planted drafts accepted by the target
    trusting = trispec_rounds(Wp, MICRO, Wt, MICRO, prompt, _mixed_drafts(Wp, MICRO, 21, 10), 6, 0.0)
    seq = trusting["sequence"]
    assert seq == greedy_decode(Wp, MICRO, prompt, len(seq) - len(prompt))
    assert not any(r["escalate"] for r in trusting["rounds"])


@pytest.mark.parametrize("lam,max_nodes,want_catch_up", [(0.25, 16, False), (0.1, 12, True)])
def test_target_catches_up_on_tokens_it_never_saw(lam, max_nodes, want_catch_up):
    """Rounds that end at the proxy leave the target's cache behind; the next escalation carries
    the unseen tokens as a forced chain (plain catch-up passes first if they do not fit), and
    afterwards both caches are the textbook caches of the emitted sequence."""
    from oracle import trispec_rounds
    Wp, Wt = _two_models(31, 32)
    prompt = gen_context_tokens(MICRO.vocab, 5, 31).tolist()
    drafts = _mixed_drafts(Wp, MICRO, 31, 10)
    # a threshold in the middle of the proxy's margins: some rounds end at the proxy, some escalate
    res = trispec_rounds(Wp, MICRO, Wt, MICRO, prompt, drafts, 14, lam, max_nodes=max_nodes)
    esc = [r["escalate"] for r in res["rounds"]]
    assert 0 < sum(esc) < len(esc)
    carried = any(r["escalate"] and r["n_forced_t"] > len(r["proxy"]["path"]) for r in res["rounds"])
    caught_up = any(r["catch_up"] > 0 for r in res["rounds"])
    assert caught_up == want_catch_up and (carried or caught_up)      # the lag went in one way or the other
    assert all(r["target_nodes"] <= max_nodes for r in res["rounds"] if r["escalate"])
    seq = res["sequence"]
    refp = causal_forward(Wp, MICRO, seq[:-1])
    assert np.max(np.abs(res["kp"] - refp["K"])) < 1e-9 and np.max(np.abs(res["vp"] - refp["V"])) < 1e-9
    t_len = res["kt"].shape[2]
    reft = causal_forward(Wt, MICRO, seq[:t_len])
    assert np.max(np.abs(res["kt"] - reft["K"])) < 1e-9 and np.max(np.abs(res["vt"] - reft["V"])) < 1e-9


# ------------------------------------------------------------------ sampling rounds (Alg. 1 as printed)
def _self_drafter(Wd, shape, k, temperature, seed, noise=0.0, one_hot=False):
    """A drafter that is itself a model: x_i drawn from softmax(logits_d / T) (plus optional
    noise on its logits), autoregressively, with numpy's generator; reports those distributions."""
    from oracle import tempered_softmax

    def fn(r, seq, _cache_len):
        rng = np.random.default_rng(seed * 1000 + r)
        cur = list(seq)
        toks, rows = [0], []
        for _ in range(k):
            lg = causal_forward(Wd, shape, cur, last_only=True)["logits"][0]
            q = tempered_softmax(lg + noise * rng.standard_normal(lg.shape), temperature)
            x = int(rng.choice(len(q), p=q))
            if one_hot:
                x = int(np.argmax(q)) if rng.random() < 0.7 else x
                q = np.eye(len(q))[x]
            toks.append(x); rows.append(q); cur.append(x)
        return {"tokens": np.array(toks, dtype=np.int32), "p_draft": np.stack(rows),
                "u_accept_p": rng.random(k + 1), "u_sample_p": rng.random(),
                "u_accept_t": rng.random(k + 1), "u_sample_t": rng.random()}
    return fn


def test_sampling_rounds_reduce_to_the_greedy_rounds_at_low_temperature():
    """One-hot drafts and T -> 0: Eq. 6 is the indicator, so the sampling rounds must emit what the
    (separately pinned) greedy rounds emit for the same drafts, round for round."""
    from oracle import CRIT_TOP1, trispec_rounds, trispec_sample_rounds
    Wp, Wt = _two_models(41, 42)
    prompt = gen_context_tokens(MICRO.vocab, 5, 41).tolist()
    drafts = _self_drafter(Wp, MICRO, 4, 1.0, 41, one_hot=True)
    log = {}

    def same_drafts_as_tree(r, seq):
        d = drafts(r, seq, 0)
        log[r] = d
        return gen_chain(5), d["tokens"]
    # only thresholds on which the trust predicate cannot differ: it is evaluated on the tempered
    # distribution, whose top-1 probability tends to 1 as T -> 0
    for lam in (0.0, 2.0):
        greedy = trispec_rounds(Wp, MICRO, Wt, MICRO, prompt, same_drafts_as_tree, 6, lam, CRIT_TOP1)
        sampled = trispec_sample_rounds(Wp, MICRO, Wt, MICRO, prompt, lambda r, s, c: log[r], 6, lam, 1e-3,
                                        CRIT_TOP1)
        assert sampled["sequence"] == greedy["sequence"], lam
        assert [r["escalate"] for r in sampled["rounds"]] == [r["escalate"] for r in greedy["rounds"]]


def test_sampling_rounds_are_lossless_when_the_proxy_is_never_trusted():
    """lambda > 1: every round escalates at the root and the target decides by speculative sampling,
    so the first emitted token follows the TARGET's tempered distribution exactly (Sec. 2.1), whatever
    the proxy and the drafter are.  Monte Carlo over numpy's generator on the 61-token micro model."""
    from oracle import tempered_softmax, trispec_sample_rounds
    Wp, Wt = _two_models(51, 52)
    prompt = gen_context_tokens(MICRO.vocab, 4, 51).tolist()
    T, N = 0.9, 2500
    p_t = tempered_softmax(causal_forward(Wt, MICRO, prompt, last_only=True)["logits"][0], T)
    counts = np.zeros(MICRO.vocab)
    lens = []
    for n in range(N):
        res = trispec_sample_rounds(Wp, MICRO, Wt, MICRO, prompt, _self_drafter(Wp, MICRO, 2, T, 7000 + n, noise=0.5),
                                    1, 2.0, T)
        assert res["rounds"][0]["escalate"] == 1 and res["rounds"][0]["proxy"]["accepted_len"] == 0
        counts[res["sequence"][len(prompt)]] += 1
        lens.append(len(res["sequence"]) - len(prompt))
    big = p_t > 5.0 / N
    chi2 = float(((counts[big] - N * p_t[big]) ** 2 / (N * p_t[big])).sum())
    dof = int(big.sum()) - 1
    assert chi2 < dof + 5 * np.sqrt(2 * dof), (chi2, dof)
    assert 1.0 < np.mean(lens) < 3.0          # some drafts were accepted by the target, not all


def test_sampling_rounds_with_a_perfect_drafter_accept_everything_and_keep_textbook_caches():
    from oracle import trispec_sample_rounds
    W = oracle_weights(MICRO, 61)
    prompt = gen_context_tokens(MICRO.vocab, 5, 61).tolist()
    T, k = 0.8, 3
    res = trispec_sample_rounds(W, MICRO, W, MICRO, prompt, _self_drafter(W, MICRO, k, T, 61), 5, 0.0, T)
    for r in res["rounds"]:        # p_d = p_v: ratio 1, every uniform accepts; margin >= 0 never escalates
        assert r["escalate"] == 0 and r["proxy"]["accepted_len"] == k and r["proxy"]["row"] == k
    seq = res["sequence"]
    assert len(seq) == len(prompt) + 5 * (k + 1)
    ref = causal_forward(W, MICRO, seq[:-1])
    assert np.max(np.abs(res["kp"] - ref["K"])) < 1e-9 and np.max(np.abs(res["vp"] - ref["V"])) < 1e-9


@pytest.mark.parametrize("max_nodes", [16, 8])
def test_sampling_rounds_mixed_routing_keeps_both_caches_textbook(max_nodes):
    from oracle import trispec_sample_rounds
    Wp, Wt = _two_models(71, 72)
    prompt = gen_context_tokens(MICRO.vocab, 5, 71).tolist()
    res = trispec_sample_rounds(Wp, MICRO, Wt, MICRO, prompt, _self_drafter(Wp, MICRO, 3, 0.7, 71, noise=0.8), 14,
                                0.12, 0.7, max_nodes=max_nodes)
    esc = [r["escalate"] for r in res["rounds"]]
    assert 0 < sum(esc) < len(esc)
    assert any(r["escalate"] and r["u"] > 0 for r in res["rounds"]) or any(r["catch_up"] for r in res["rounds"])
    assert all(r["target_nodes"] <= max_nodes for r in res["rounds"] if r["escalate"])
    seq = res["sequence"]
    refp = causal_forward(Wp, MICRO, seq[:-1])
    assert np.max(np.abs(res["kp"] - refp["K"])) < 1e-9 and np.max(np.abs(res["vp"] - refp["V"])) < 1e-9
    t_len = res["kt"].shape[2]
    reft = causal_forward(Wt, MICRO, seq[:t_len])
    assert np.max(np.abs(res["kt"] - reft["K"])) < 1e-9 and np.max(np.abs(res["vt"] - reft["V"])) < 1e-9
