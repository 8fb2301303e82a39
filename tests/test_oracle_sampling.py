"""Pins of the sampling-mode decision oracle against what Sec. 2.1 / Eq. 6 and the mathematics
fix: the exactness theorem of speculative sampling (the emitted token is distributed as the
verifier's own distribution) enumerated exactly and checked by Monte Carlo with numpy's
generator, the greedy limit the paper states below Eq. 6, exact interval counts of the
inverse CDF, and the degenerate cases."""
import numpy as np
import pytest

from oracle import CRIT_MARGIN, CRIT_TOP1, decide, node_stats
from oracle.sampling import (RESAMPLE_DIRECT, RESAMPLE_RESIDUAL, accept_probability, inverse_cdf,
                             residual_distribution, residual_mass, sample_decide, tempered_softmax)


def _dist(rng, V, zeros=0):
    p = rng.dirichlet(np.ones(V) * 0.7)
    if zeros:
        p[rng.choice(V, zeros, replace=False)] = 0.0
        p /= p.sum()
    return p


@pytest.mark.parametrize("seed", range(6))
def test_one_step_is_exactly_the_verifier_distribution(seed):
    """sum_x q(x) [a(x) 1{y = x} + (1 - a(x)) res(y)] = p(y): exact enumeration (Sec. 2.1, lossless)."""
    rng = np.random.default_rng(seed)
    V = 7
    p, q = _dist(rng, V, zeros=seed % 2), _dist(rng, V, zeros=(seed // 2) % 2)
    res = residual_distribution(p, q)
    out = np.zeros(V)
    for x in range(V):
        if q[x] == 0:
            continue
        a = accept_probability(p, q, x)
        out[x] += q[x] * a
        out += q[x] * (1 - a) * res
    assert np.allclose(out, p, atol=1e-13)
    assert np.all(residual_mass(p, q) >= 0) and residual_mass(p, q)[p <= q].sum() == 0


def test_accept_probability_values():
    p, q = np.array([0.5, 0.25, 0.25, 0.0]), np.array([0.25, 0.5, 0.0, 0.25])
    assert accept_probability(p, q, 0) == 1.0          # p > q
    assert accept_probability(p, q, 1) == 0.5          # p / q
    assert accept_probability(p, q, 2) == 1.0          # q = 0 < p
    assert accept_probability(p, q, 3) == 0.0          # p = 0
    assert np.allclose(residual_distribution(p, q), [0.5, 0, 0.5, 0])


def test_tempered_softmax_closed_forms():
    l = np.log(np.array([1.0, 2.0, 4.0, 1.0]))
    assert np.allclose(tempered_softmax(l, 1.0), np.array([1, 2, 4, 1]) / 8)
    assert np.allclose(tempered_softmax(l, 0.5), np.array([1, 4, 16, 1]) / 22)        # p^(1/T)
    assert np.allclose(tempered_softmax(l + 1000.0, 2.0), np.sqrt([1, 2, 4, 1]) / np.sqrt([1, 2, 4, 1]).sum())


def test_inverse_cdf_interval_counts_are_exact():
    mass = np.array([0, 3, 0, 5, 1, 0, 7, 0]) / 4.0          # total 4: not normalised on purpose
    n = 1600
    counts = np.bincount([inverse_cdf(mass, (j + 0.5) / n) for j in range(n)], minlength=8)
    assert counts.tolist() == [0, 300, 0, 500, 100, 0, 700, 0]
    assert inverse_cdf(mass, 0.0) == 1                        # first token with mass
    assert inverse_cdf(mass, np.nextafter(1.0, 0.0)) == 6     # last token with mass
    assert inverse_cdf(mass, 3 / 16) == 3                     # boundaries belong to the upper interval


def _table_model(rng, V):
    """p(. | prefix) and q(. | prefix) for prefixes of length 0, 1, 2 over a tiny vocabulary."""
    p0, q0 = _dist(rng, V), _dist(rng, V)
    p1 = np.stack([_dist(rng, V) for _ in range(V)]); q1 = np.stack([_dist(rng, V) for _ in range(V)])
    p2 = np.stack([[_dist(rng, V) for _ in range(V)] for _ in range(V)])
    return p0, q0, p1, q1, p2


@pytest.mark.parametrize("resample", [RESAMPLE_RESIDUAL, RESAMPLE_DIRECT])
def test_monte_carlo_two_token_chain_matches_the_verifier(resample):
    """Drafts drawn from q by numpy's generator, then the whole walk.  With the residual rule the
    first emitted token follows p(.) and, given a first accepted token x, the second emitted one
    follows p(. | x) — which fails if the walk reads the wrong row of the logits, of the draft
    table or of the uniforms.  The direct rule is biased exactly as the enumeration predicts."""
    rng = np.random.default_rng(11)
    V, N = 5, 60000
    p0, q0, p1, q1, p2 = _table_model(rng, V)
    first = np.zeros(V)
    second = np.zeros((V, V))
    lens = np.zeros(3)
    for _ in range(N):
        x1 = int(rng.choice(V, p=q0)); x2 = int(rng.choice(V, p=q1[x1]))
        logits = np.log(np.stack([p0, p1[x1], p2[x1][x2]])) + rng.normal()     # softmax is shift-invariant
        o = sample_decide(logits, [0, x1, x2], np.stack([q0, q1[x1]]), rng.random(3), rng.random(),
                          temperature=1.0, lam=0.0, resample=resample)
        emitted = [x1, x2][:o["accepted_len"]] + [o["token"]]
        assert o["escalate"] == 0 and o["path"] == list(range(o["accepted_len"] + 1))
        assert o["row"] == o["accepted_len"]
        lens[o["accepted_len"]] += 1
        first[emitted[0]] += 1
        if o["accepted_len"] >= 1:
            second[emitted[0], emitted[1]] += 1
    if resample == RESAMPLE_RESIDUAL:
        want_first = p0
    else:   # accepted mass min(p, q), the rest of the probability redistributed as p
        acc = np.minimum(p0, q0)
        want_first = acc + (1 - acc.sum()) * p0
    assert np.all(np.abs(first / N - want_first) < 5 * np.sqrt(want_first * (1 - want_first) / N) + 1e-9)
    assert abs(lens[0] / N - (1 - np.minimum(p0, q0).sum())) < 0.01             # P(reject first) = TV distance
    if resample == RESAMPLE_RESIDUAL:
        for x in range(V):
            n = second[x].sum()
            if n < 2000:
                continue
            assert np.all(np.abs(second[x] / n - p1[x]) < 5 * np.sqrt(p1[x] * (1 - p1[x]) / n) + 1e-9), x


def test_greedy_limit_equals_the_greedy_decision():
    """Below Eq. 6: with one-hot distributions the Bernoulli variable is 1{x_p = x_d}.  A tiny
    temperature and one-hot draft distributions must reproduce the greedy walk for any uniforms."""
    rng = np.random.default_rng(5)
    V, M = 9, 6
    for trial in range(40):
        logits = rng.normal(size=(M, V)) * 3
        st = node_stats(logits)
        tokens = rng.integers(0, V, M)
        good = int(rng.integers(0, M))                      # drafts follow the verifier for `good` steps
        for i in range(1, good + 1):
            tokens[i] = st["argmax"][i - 1]
        q = np.zeros((M - 1, V)); q[np.arange(M - 1), tokens[1:]] = 1.0
        for n_forced in (1, 2):
            want = decide(tokens, np.arange(-1, M - 1), st["argmax"], st["conf"], st["margin"], 0.0,
                          CRIT_TOP1, n_forced)
            got = sample_decide(logits, tokens, q, rng.random(M) * 0.999, rng.random() * 0.999, 1e-3, 0.0,
                                CRIT_TOP1, n_forced)
            assert (got["accepted_len"], got["token"], got["escalate"]) == \
                (want["accepted_len"], want["token"], want["escalate"]), (trial, n_forced)
            assert got["path"] == list(want["path"])


def test_equal_distributions_accept_everything_and_bonus_is_direct():
    rng = np.random.default_rng(2)
    V, M = 8, 5
    logits = rng.normal(size=(M, V))
    p = tempered_softmax(logits, 0.7)
    tokens = rng.integers(0, V, M)
    o = sample_decide(logits, tokens, p[:-1], np.full(M, 0.999999), 0.4, 0.7, 0.0)
    assert o["accepted_len"] == M - 1 and o["row"] == M - 1 and o["escalate"] == 0
    assert o["token"] == inverse_cdf(p[-1], 0.4)


def test_forced_prefix_is_never_tested_and_routing_follows_the_threshold():
    rng = np.random.default_rng(3)
    V, M = 8, 6
    logits = rng.normal(size=(M, V))
    tokens = rng.integers(0, V, M)
    p = tempered_softmax(logits, 1.0)
    q = np.stack([_dist(rng, V) for _ in range(M - 1)])
    u = np.full(M, 0.999999)                        # rejects whatever has ratio < 1
    q[2] = p[2]                                     # node 3 is certain to pass
    for i in (0, 1):                                # nodes 1, 2 certain to fail if tested
        q[i] = np.eye(V)[tokens[i + 1]] * 0.9 + 0.1 / V
        assert p[i][tokens[i + 1]] < 0.9
    q[3] = np.eye(V)[tokens[4]] * 0.9 + 0.1 / V
    o = sample_decide(logits, tokens, q, u, 0.3, 1.0, 0.0, n_forced=3)
    assert o["path"] == [2, 3] and o["accepted_len"] == 1 and o["row"] == 3
    assert sample_decide(logits, tokens, q, u, 0.3, 1.0, 0.0, n_forced=1)["accepted_len"] == 0
    # lambda above 1 escalates at the first node whatever the uniforms; accepted_len is monotone in lambda
    esc = sample_decide(logits, tokens, p[:-1], u * 0, 0.3, 1.0, 1.5)
    assert (esc["accepted_len"], esc["token"], esc["escalate"], esc["row"]) == (0, -1, 1, -1)
    prev = M
    for lam in (0.0, 0.05, 0.1, 0.2, 0.4, 0.8, 1.1):
        o = sample_decide(logits, tokens, p[:-1], u * 0, 0.3, 1.0, lam, CRIT_MARGIN)
        assert o["accepted_len"] <= prev
        prev = o["accepted_len"]
        srt = np.sort(p, axis=1)
        margins = srt[:, -1] - srt[:, -2]
        first_untrusted = next((i for i in range(M) if margins[i] < lam), M)
        assert o["escalate"] == (1 if first_untrusted < M else 0)
        assert o["accepted_len"] == min(first_untrusted, M - 1)
