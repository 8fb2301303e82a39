"""Pins for the oracle's decision rule: the set-min definitions of tau_a / tau_m exactly as
printed (paper Eq. 7, Eq. 9), the two routing cases (Sec. 3.2), and the invariants."""
import itertools

import numpy as np
import pytest

from oracle import (CRIT_MARGIN, CRIT_TOP1, chain_round_output, chain_tau_a, chain_tau_m, decide,
                    node_stats, prune_reroot, tie_flags, verify_forward)
from workloads import gen_chain, gen_context_tokens, gen_draft_tokens, gen_tree, tree_depths
from helpers import MICRO, oracle_weights, path_to, prefill


def test_printed_definitions_by_hand():
    # k = 3. s = (1,1,0): first rejection at draft 3 -> tau_a = 2.  all accepted -> k.
    assert chain_tau_a([1, 1, 0]) == 2 and chain_tau_a([1, 1, 1]) == 3 and chain_tau_a([0, 1, 1]) == 0
    # g over p_1..p_4: first untrusted distribution p_2 -> tau_m = 1; all trusted -> k+1 (Sec. 3.2)
    assert chain_tau_m([1, 0, 1, 1]) == 1 and chain_tau_m([1, 1, 1, 1]) == 4 and chain_tau_m([0, 1, 1, 1]) == 0
    # Case I: tau_a < tau_m, output x_1..x_tau_a + proxy token of position tau_a+1
    assert chain_round_output([1, 1, 0], [1, 1, 1, 1]) == (1, 2, 3)
    # Case II on equality (tau_a >= tau_m)
    assert chain_round_output([1, 1, 0], [1, 1, 0, 1]) == (2, 2, 0)
    assert chain_round_output([1, 1, 1], [1, 1, 1, 1]) == (1, 3, 4)   # all accepted + bonus from p_{k+1}
    assert chain_round_output([1, 1, 1], [1, 1, 1, 0]) == (2, 3, 0)


@pytest.mark.parametrize("k", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("criterion", [CRIT_MARGIN, CRIT_TOP1])
def test_walk_equals_set_min_definitions_exhaustively(k, criterion):
    """Every (s, g) pattern on a chain of k drafts: the tree walk must reproduce Eq. 7 / Eq. 9
    and the Case I / Case II outputs."""
    lam = 0.5
    parents = gen_chain(k + 1)
    for s in itertools.product([0, 1], repeat=k):
        for g in itertools.product([0, 1], repeat=k + 1):
            tokens = np.arange(100, 101 + k)                    # node j carries token 100+j
            # verifier's argmax at node j is the token it predicts for position j+1
            argmax = np.array([(101 + j) if (j < k and s[j]) else 7 for j in range(k + 1)])
            stat = np.array([0.9 if gj else 0.1 for gj in g])
            conf = stat if criterion == CRIT_TOP1 else np.full(k + 1, 0.95)
            margin = stat if criterion == CRIT_MARGIN else np.full(k + 1, 0.0)
            got = decide(tokens, parents, argmax, conf, margin, lam, criterion)
            case, acc, src = chain_round_output(s, g)
            assert got["accepted_len"] == acc
            assert got["escalate"] == (1 if case == 2 else 0)
            assert got["path"] == list(range(acc + 1))
            if case == 1:
                assert got["token"] == argmax[src - 1]          # p_{src} is emitted at node src-1
            else:
                assert got["token"] == -1
            assert acc == min(chain_tau_a(s), chain_tau_m(g))


def test_threshold_boundary_is_inclusive():
    parents = gen_chain(2)
    out = decide([5, 6], parents, [6, 9], [0.5, 0.5], [0.5, 0.5], 0.5, CRIT_MARGIN)
    assert out["escalate"] == 0 and out["accepted_len"] == 1 and out["token"] == 9
    out = decide([5, 6], parents, [6, 9], [0.5, 0.5], [0.5 - 1e-12, 0.5], 0.5, CRIT_MARGIN)
    assert out["escalate"] == 1 and out["accepted_len"] == 0


def test_tree_walk_picks_matching_child_and_lowest_duplicate():
    #      0
    #    / | \
    #   1  2  3      tokens 1:40 2:41 3:41 (duplicate siblings), 4 under 2, 5 under 3
    parents = np.array([-1, 0, 0, 0, 2, 3])
    tokens = np.array([9, 40, 41, 41, 50, 50])
    argmax = np.array([41, 0, 50, 50, 77, 78])
    ones = np.ones(6)
    out = decide(tokens, parents, argmax, ones, ones, 0.5)
    assert out["path"] == [0, 2, 4] and out["accepted_len"] == 2 and out["token"] == 77 and out["escalate"] == 0
    # forced prefix: walk starts at node n_forced-1 and does not count forced nodes
    parents = np.array([-1, 0, 1, 2, 2])
    tokens = np.array([9, 10, 11, 60, 61])
    argmax = np.array([0, 0, 61, 5, 6])
    out = decide(tokens, parents, argmax, np.ones(5), np.ones(5), 0.5, n_forced=3)
    assert out["path"] == [2, 4] and out["accepted_len"] == 1 and out["token"] == 6


def _micro_case(seed, C=8, M=14):
    shape = MICRO
    W = oracle_weights(shape, seed)
    ctx = gen_context_tokens(shape.vocab, C, seed)
    Kc, Vc = prefill(shape, seed, ctx)
    parents = gen_tree(M, 5, 3, seed)
    toks = gen_draft_tokens(parents, shape.vocab, seed)
    return shape, W, Kc, Vc, parents, toks, C


def _plant_greedy_path(shape, W, Kc, Vc, parents, toks, C, leaf):
    """Overwrite tokens along root->leaf with the verifier's own greedy continuation."""
    toks = toks.copy()
    pos = C + tree_depths(parents)
    p = path_to(parents, leaf)
    for a, b in zip(p[:-1], p[1:]):
        st = node_stats(verify_forward(W, shape, Kc, Vc, toks, parents, pos)["logits"])
        toks[b] = st["argmax"][a]
    return toks


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_invariants_on_model_outputs(seed):
    shape, W, Kc, Vc, parents, toks, C = _micro_case(seed)
    depth = tree_depths(parents)
    leaf = int(np.argmax(depth))
    toks = _plant_greedy_path(shape, W, Kc, Vc, parents, toks, C, leaf)
    st = node_stats(verify_forward(W, shape, Kc, Vc, toks, parents, C + depth)["logits"])
    for crit in (CRIT_MARGIN, CRIT_TOP1):
        # lambda = 0: everything trusted; drafts = own greedy continuation -> whole path accepted
        out = decide(toks, parents, st["argmax"], st["conf"], st["margin"], 0.0, crit)
        assert out["escalate"] == 0 and out["accepted_len"] == depth[leaf]
        assert out["path"] == path_to(parents, leaf) and out["token"] == st["argmax"][leaf]
        # lambda > 1: nothing trusted
        out = decide(toks, parents, st["argmax"], st["conf"], st["margin"], 1.5, crit)
        assert out["escalate"] == 1 and out["accepted_len"] == 0 and out["token"] == -1
        # monotone in lambda; never deeper than the tree
        prev_acc, prev_esc = 10 ** 9, 0
        for lam in np.linspace(0, 1.01, 40):
            out = decide(toks, parents, st["argmax"], st["conf"], st["margin"], lam, crit)
            assert out["accepted_len"] <= prev_acc and out["escalate"] >= prev_esc
            assert out["accepted_len"] <= depth.max()
            prev_acc, prev_esc = out["accepted_len"], out["escalate"]


def test_tie_flags():
    st = {"margin": np.array([0.5004, 0.2, 0.9]), "conf": np.array([0.7, 0.3, 0.95]),
          "l1": np.array([3.0, 2.0, 1.0]), "l2": np.array([1.0, 1.9995, -4.0])}
    assert list(tie_flags(st, 0.5, CRIT_MARGIN)) == [True, True, False]
    assert list(tie_flags(st, 0.3, CRIT_TOP1)) == [False, True, False]


@pytest.mark.parametrize("seed", [0, 3])
def test_prune_reroot_keeps_the_subtree_and_its_logits(seed):
    shape, W, Kc, Vc, parents, toks, C = _micro_case(seed, M=16)
    depth = tree_depths(parents)
    pos = C + depth
    full = verify_forward(W, shape, Kc, Vc, toks, parents, pos)["logits"]
    for last in range(len(parents)):
        path = path_to(parents, last)
        pr = prune_reroot(toks, parents, pos, path)
        kept = list(pr["old_id"])
        # brute force: kept = path + strict descendants of `last`
        want = path + [i for i in range(len(parents)) if last in path_to(parents, i)[:-1]]
        assert kept == want and pr["n_forced"] == len(path)
        assert list(pr["parents"][: len(path)]) == list(range(-1, len(path) - 1))
        assert np.array_equal(pr["positions"], pos[kept]) and np.array_equal(pr["tokens"], toks[kept])
        for j, old in enumerate(kept):
            if j > 0:
                assert kept[pr["parents"][j]] == parents[old]
        # a node's distribution depends only on its ancestors, all of which were kept (Eq. 10)
        sub = verify_forward(W, shape, Kc, Vc, pr["tokens"], pr["parents"], pr["positions"])["logits"]
        assert np.max(np.abs(sub - full[kept])) < 1e-10
        # target-side walk on the pruned tree == walk on the full tree started below `last`
        st_full, st_sub = node_stats(full), node_stats(sub)
        a = decide(pr["tokens"], pr["parents"], st_sub["argmax"], st_sub["conf"], st_sub["margin"], 0.0,
                   n_forced=pr["n_forced"])
        cur, acc = last, 0
        while True:
            nxt = [c for c in range(len(parents)) if parents[c] == cur and toks[c] == st_full["argmax"][cur]]
            if not nxt:
                break
            cur, acc = nxt[0], acc + 1
        assert a["accepted_len"] == acc and a["token"] == st_full["argmax"][cur] and a["escalate"] == 0
        assert [kept[j] for j in a["path"]] == path_to(parents, cur)[len(path) - 1:]


def test_tie_resolutions_enumerate_the_other_outcomes():
    """The helper the GPU tests use to excuse a tie: on a chain whose statistic at node 1 sits on the
    threshold and whose top two logits at node 2 are equal within the tolerance, the enumerated
    decisions are exactly the four outcomes of resolving the two ties either way."""
    from types import SimpleNamespace
    from gpu_helpers import tie_resolutions
    from oracle import CRIT_TOP1, node_stats
    V = 11
    logits = np.full((4, V), -5.0)
    logits[0, 3] = 5.0                       # node 0: confident, argmax 3
    logits[1, 4] = 0.0; logits[1, 5] = -0.1; logits[1, 9] = -0.2  # node 1: argmax 4, top-1 probability near 0.36
    logits[2, 6] = 1.0; logits[2, 7] = 1.0 - 5e-4   # node 2: top two within 1e-3
    logits[3, 8] = 4.0
    st = node_stats(logits)
    lam = float(st["conf"][1]) + 4e-4        # node 1's statistic within 1e-3 below the threshold
    tokens = np.array([[0, 3, 4, 7]], dtype=np.int32)    # chain 0 -> 1 -> 2 -> 3; node 3 holds the RUNNER-UP of node 2
    parents = np.array([[-1, 0, 1, 2]], dtype=np.int32)
    case = SimpleNamespace(tokens=tokens, parents=parents)
    out = [{"stats": st, "logits": logits}]
    alts = tie_resolutions(case, out, 0, lam, CRIT_TOP1, 1, [1, 2])
    got = sorted((a["accepted_len"], a["token"], a["escalate"]) for a in alts)
    # node 1 untrusted -> escalate after 1 draft (twice: node 2's tie no longer matters);
    # node 1 trusted, node 2's argmax 6 -> no child matches: stop after 2 with token 6;
    # node 1 trusted, node 2's argmax 7 -> node 3 accepted, then node 3's own argmax 8 as the bonus
    assert got == sorted([(1, -1, 1), (1, -1, 1), (2, 6, 0), (3, 8, 0)]), got


# ---- entropy statistic / criterion and the top-k rank of the appendix's relaxed verification

def test_entropy_closed_forms_and_library():
    from scipy.special import softmax
    from scipy.stats import entropy as scipy_entropy
    from oracle import node_stats
    V = 1000
    rng = np.random.default_rng(5)
    uniform = np.zeros((1, V))
    assert abs(node_stats(uniform)["entropy"][0] - np.log(V)) < 1e-12
    one_hot = np.full((1, V), -1e4); one_hot[0, 17] = 0.0
    assert node_stats(one_hot)["entropy"][0] == 0.0                     # exp underflows to exactly 0: 0 ln 0 = 0
    two = np.full((1, V), -np.inf); two[0, 3] = np.log(0.25); two[0, 900] = np.log(0.75)
    assert abs(node_stats(two)["entropy"][0] - (-(0.25 * np.log(0.25) + 0.75 * np.log(0.75)))) < 1e-12
    logits = rng.standard_normal((7, V)) * 4
    got = node_stats(logits)["entropy"]
    assert np.allclose(got, scipy_entropy(softmax(logits, axis=1), axis=1), rtol=0, atol=1e-12)
    assert np.all(got >= 0) and np.all(got <= np.log(V) + 1e-12)
    assert np.allclose(node_stats(logits + 123.0)["entropy"], got, atol=1e-10)     # shift invariance
    # k equal maxima far above the rest: H = ln k
    flat3 = np.full((1, V), -1e4); flat3[0, [1, 50, 700]] = 2.0
    assert abs(node_stats(flat3)["entropy"][0] - np.log(3)) < 1e-12


def test_entropy_criterion_in_the_walk():
    """g = 1{H <= lambda}: lambda = ln V trusts every node, lambda < 0 none; in between exactly the
    nodes whose entropy is at most lambda, so on a chain tau_m is the first node above it."""
    from oracle import CRIT_ENTROPY, decide, node_stats
    rng = np.random.default_rng(6)
    V, M = 50, 7
    logits = rng.standard_normal((M, V)) * rng.uniform(0.5, 6, (M, 1))
    st = node_stats(logits)
    tokens = np.concatenate([[0], st["argmax"][:-1]]).astype(np.int32)       # every draft is the greedy token
    parents = np.arange(-1, M - 1)
    kw = dict(entropy=st["entropy"])
    d = decide(tokens, parents, st["argmax"], st["conf"], st["margin"], np.log(V), CRIT_ENTROPY, 1, **kw)
    assert (d["accepted_len"], d["escalate"]) == (M - 1, 0)
    d = decide(tokens, parents, st["argmax"], st["conf"], st["margin"], -0.1, CRIT_ENTROPY, 1, **kw)
    assert (d["accepted_len"], d["escalate"], d["token"]) == (0, 1, -1)
    for lam in np.sort(st["entropy"])[:-1] + 1e-9:
        d = decide(tokens, parents, st["argmax"], st["conf"], st["margin"], lam, CRIT_ENTROPY, 1, **kw)
        above = np.nonzero(st["entropy"] > lam)[0]
        assert d["escalate"] == 1 and d["accepted_len"] == above[0]


def test_draft_ranks_against_a_sort_and_the_top_k_walk():
    from oracle import decide, draft_ranks, node_stats
    from workloads import gen_tree
    rng = np.random.default_rng(7)
    V, M = 40, 25
    parents = gen_tree(M, 6, 3, 7)
    logits = np.round(rng.standard_normal((M, V)) * 2, 1)                 # rounded: equal logits do occur
    tokens = rng.integers(0, V, M).astype(np.int32)
    ranks = draft_ranks(logits, tokens, parents)
    assert ranks[0] == -1
    for i in range(1, M):
        order = np.argsort(-logits[parents[i]], kind="stable")            # descending logit, ties by token id
        assert order[ranks[i]] == tokens[i]
    st = node_stats(logits)
    # top_k = 1 is the greedy walk; top_k = V accepts the first child of every node down to a leaf
    a = decide(tokens, parents, st["argmax"], st["conf"], st["margin"], 0.0, 0, 1)
    tok1 = tokens.copy()
    b = decide(tok1, parents, st["argmax"], st["conf"], st["margin"], 0.0, 0, 1, ranks=ranks, top_k=1)
    assert a == b
    c = decide(tokens, parents, st["argmax"], st["conf"], st["margin"], 0.0, 0, 1, ranks=ranks, top_k=V)
    cur, n = 0, 0
    while True:
        kids = [j for j in range(M) if parents[j] == cur]
        if not kids:
            break
        cur, n = kids[0], n + 1
    assert c["accepted_len"] == n and c["path"][-1] == cur and c["token"] == st["argmax"][cur]
    # monotone in k: a larger k never shortens the accepted prefix of a CHAIN
    chain = np.arange(-1, M - 1)
    rk = draft_ranks(logits, tokens, chain)
    lens = [decide(tokens, chain, st["argmax"], st["conf"], st["margin"], 0.0, 0, 1, ranks=rk, top_k=k)["accepted_len"]
            for k in (1, 2, 4, 8, 16, V)]
    assert lens == sorted(lens) and lens[-1] == M - 1
    assert lens[1] == next((i for i in range(1, M) if rk[i] >= 2), M) - 1
