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
