"""Sampling-mode chain decision (Sec. 2.1 acceptance + residual resampling, Eq. 6 - Eq. 9 routing)
on the GPU against the fp64 oracle.  Integer outputs must be equal; a sequence is excused only when
the oracle itself says a comparison sits within rounding of its boundary (u * p_d(x) against p_v(x),
a statistic against the threshold), and a sampled token only when u * total lies within `eps` of
the boundary of the interval the GPU chose."""
import numpy as np
import pytest
import torch

from gpu_helpers import Case, device_model
from helpers import prefill
from oracle import CRIT_MARGIN, CRIT_TOP1, RESAMPLE_DIRECT, RESAMPLE_RESIDUAL, inverse_cdf, tempered_softmax
from oracle import sample_decide as oracle_sample_decide
from paper_2601_23180_amd import sample_decide
from workloads import SHAPES, gen_chain, gen_context_tokens, gen_draft_distributions, gen_uniforms, tree_depths

pytestmark = pytest.mark.gpu


def run_gpu(logits, tokens, p_draft, ua, us, T, lam, crit, n_forced, resample):
    dev = lambda x, dt: torch.from_numpy(np.ascontiguousarray(x)).to(dt).cuda()
    out = sample_decide(dev(logits, torch.float32), dev(tokens, torch.int32), dev(p_draft, torch.float32),
                        dev(ua, torch.float32), dev(us, torch.float32), T, lam, crit, n_forced, resample)
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in out.items() if not k.startswith("_")}


def compare(logits, tokens, p_draft, ua, us, T, lam, crit, n_forced, resample, got, eps, tol_stat):
    """Returns (sequences compared in full, sequences excused, tokens excused)."""
    B, M, V = logits.shape
    full = excused = tok_excused = 0
    assert got["status"][0] == 0
    for b in range(B):
        o = oracle_sample_decide(logits[b], tokens[b], p_draft[b], ua[b], float(us[b]), T, lam, crit, n_forced, resample)
        p = tempered_softmax(logits[b], T)
        srt = np.sort(p, axis=1)
        conf, margin = srt[:, -1], srt[:, -1] - (srt[:, -2] if V > 1 else 0.0)
        assert np.allclose(got["confidence"][b, :M], conf, rtol=tol_stat, atol=1e-7)
        assert np.allclose(got["margin"][b, :M], margin, rtol=0, atol=tol_stat)
        stat = margin if crit == CRIT_MARGIN else conf
        on_path = stat[o["path"]]
        # lambda <= 0 cannot flip: top-1 probability and margin are never negative on either side
        if o["slack"] < tol_stat or (lam > 0 and np.any(np.abs(on_path - lam) < tol_stat)):
            excused += 1
            continue
        full += 1
        assert int(got["accepted_len"][b]) == o["accepted_len"], (b, got["accepted_len"][b], o["accepted_len"])
        assert int(got["escalate"][b]) == o["escalate"], b
        path = got["path"][b]
        assert path[: len(o["path"])].tolist() == o["path"] and np.all(path[len(o["path"]):] == -1)
        t = int(got["token"][b])
        if t != o["token"]:
            assert o["token"] >= 0 and 0 <= t < V and o["mass"][t] > 0, (b, t, o["token"])
            c = np.cumsum(o["mass"])
            target = float(us[b]) * c[-1]
            assert (c[t - 1] if t else 0.0) - eps <= target <= c[t] + eps, (b, t, o["token"])
            tok_excused += 1
    return full, excused, tok_excused


def random_case(seed, B, M, V, T, keep=0, scale=3.0):
    rng = np.random.default_rng(seed)
    logits = (rng.standard_normal((B, M, V)) * scale).astype(np.float32)
    pd, tk = zip(*[gen_draft_distributions(logits[b], T, seed * 10 + b, keep=keep) for b in range(B)])
    ua, us = gen_uniforms(seed, B, M)
    return logits, np.stack(tk), np.stack(pd), ua, us


@pytest.mark.parametrize("V,keep", [(4096, 0), (151936, 0), (50257, 300), (1000, 20), (3, 0), (1, 0)])
@pytest.mark.parametrize("T", [0.6, 1.0, 1.7])
def test_pure_function_parity_on_random_logits(V, keep, T):
    """Same fp32 logits to both sides: only the arithmetic of the decision differs (fp32/fp64)."""
    B, M = 8, 9
    stats = np.zeros(3, dtype=int)
    lens = []
    for seed in range(3):
        logits, tokens, p_draft, ua, us = random_case(1000 * seed + V % 97, B, M, V, T, keep)
        for lam, crit, n_forced, resample in [(0.0, CRIT_MARGIN, 1, RESAMPLE_RESIDUAL), (0.0, CRIT_MARGIN, 1, RESAMPLE_DIRECT),
                                              (0.02, CRIT_MARGIN, 1, RESAMPLE_RESIDUAL), (0.3, CRIT_TOP1, 3, RESAMPLE_RESIDUAL),
                                              (0.0, CRIT_TOP1, M, RESAMPLE_RESIDUAL), (1.5, CRIT_MARGIN, 2, RESAMPLE_DIRECT)]:
            got = run_gpu(logits, tokens, p_draft, ua, us, T, lam, crit, n_forced, resample)
            stats += compare(logits, tokens, p_draft, ua, us, T, lam, crit, n_forced, resample, got, eps=2e-5, tol_stat=2e-5)
            if lam == 0.0 and n_forced == 1:
                lens.extend(got["accepted_len"].tolist())
    full, excused, tok_excused = stats
    assert excused <= 0.05 * (full + excused) and tok_excused <= 0.05 * full, stats
    if V > 3:   # the synthetic drafter is neither always nor never accepted
        assert 0 < np.mean(lens) < M - 1, np.mean(lens)


def test_no_draft_tokens_is_a_plain_draw():
    rng = np.random.default_rng(4)
    B, V = 4, 5000
    logits = (rng.standard_normal((B, 1, V)) * 2).astype(np.float32)
    ua, us = gen_uniforms(9, B, 1)
    tokens = np.zeros((B, 1), dtype=np.int32)
    got = run_gpu(logits, tokens, np.zeros((B, 0, V), dtype=np.float32), ua, us, 0.8, 0.0, CRIT_MARGIN, 1, RESAMPLE_RESIDUAL)
    full, excused, tok_excused = compare(logits, tokens, np.zeros((B, 0, V)), ua, us, 0.8, 0.0, CRIT_MARGIN, 1,
                                         RESAMPLE_RESIDUAL, got, 2e-5, 2e-5)
    assert full == B and np.all(got["accepted_len"] == 0) and np.all(got["escalate"] == 0)


def test_inverse_cdf_hits_every_token_of_a_small_vocabulary():
    """One row, uniform sweep of u: the draw visits the tokens in order, each about p(v) of the time."""
    V, n = 12, 8
    rng = np.random.default_rng(8)
    logits = rng.standard_normal((1, 1, V)).astype(np.float32)
    p = tempered_softmax(logits[0], 1.3)[0]
    seen = []
    us_all = (np.arange(n * 50) + 0.5) / (n * 50)
    for chunk in us_all.reshape(-1, n):
        lg = np.repeat(logits, n, axis=0)
        got = run_gpu(lg, np.zeros((n, 1), dtype=np.int32), np.zeros((n, 0, V), dtype=np.float32),
                      np.zeros((n, 1), dtype=np.float32), chunk.astype(np.float32), 1.3, 0.0, CRIT_MARGIN, 1, RESAMPLE_DIRECT)
        seen.extend(got["token"].tolist())
    assert seen == sorted(seen) and set(seen) == set(range(V))
    assert np.all(np.abs(np.bincount(seen, minlength=V) / len(seen) - p) <= 1.5 / len(seen) + 1e-6)


def test_invalid_token_and_massless_residual():
    rng = np.random.default_rng(6)
    B, M, V = 2, 4, 777
    logits = (rng.standard_normal((B, M, V)) * 2).astype(np.float32)
    p = np.stack([tempered_softmax(logits[b], 1.0) for b in range(B)])
    tokens = rng.integers(0, V, (B, M)).astype(np.int32)
    p_draft = (2.0 * p[:, :-1]).astype(np.float32)          # not a distribution: dominates p_v everywhere
    ua = np.full((B, M), 0.9, dtype=np.float32)             # 0.9 * 2p < p is false: reject at the first node
    us = np.array([0.25, 0.75], dtype=np.float32)
    got = run_gpu(logits, tokens, p_draft, ua, us, 1.0, 0.0, CRIT_MARGIN, 1, RESAMPLE_RESIDUAL)
    assert got["accepted_len"].tolist() == [0, 0] and got["status"][0] == 0
    for b in range(B):                                       # empty residual: falls back to a draw from p_v
        want = inverse_cdf(p[b, 0], float(us[b]))
        assert abs(int(got["token"][b]) - want) <= 1
    ua[:] = 0.4                                              # 0.4 * 2p < p: accept
    tokens[1, 2] = V + 5                                     # out of the vocabulary: reported, never accepted
    got = run_gpu(logits, tokens, p_draft, ua, us, 1.0, 0.0, CRIT_MARGIN, 1, RESAMPLE_DIRECT)
    assert got["status"][0] == 1
    assert got["accepted_len"].tolist() == [M - 1, 1]
    assert got["path"][1, :3].tolist() == [0, 1, -1]


def test_a_draw_without_usable_mass_reports_it_and_stays_in_range():
    """A NaN uniform leaves the inverse CDF without a target: the call must say so in the status word
    (bit 1) and return a token of the vocabulary (the node's argmax), not read outside the logits."""
    rng = np.random.default_rng(12)
    B, M, V = 3, 4, 9000
    logits = (rng.standard_normal((B, M, V)) * 2).astype(np.float32)
    pd, tk = zip(*[gen_draft_distributions(logits[b], 1.0, 50 + b) for b in range(B)])
    ua, us = gen_uniforms(5, B, M)
    us = us.copy()
    us[1] = np.nan
    got = run_gpu(logits, np.stack(tk), np.stack(pd), ua, us, 1.0, 0.0, CRIT_MARGIN, 1, RESAMPLE_RESIDUAL)
    assert got["status"][0] == 2
    assert np.all((got["token"] >= 0) & (got["token"] < V))
    row = int(got["accepted_len"][1])
    assert int(got["token"][1]) == int(np.argmax(logits[1, row]))
    us[1] = 0.5                                               # the same call with a proper uniform: clean status
    got = run_gpu(logits, np.stack(tk), np.stack(pd), ua, us, 1.0, 0.0, CRIT_MARGIN, 1, RESAMPLE_RESIDUAL)
    assert got["status"][0] == 0


@pytest.mark.parametrize("key,tol", [("tiny", 3e-4), ("tiny_bf16", 5e-3)])
def test_after_a_real_verification_pass(key, tol):
    """Logits from trispec_verify on a chain, decision from trispec_sample_decide; the oracle runs its
    own fp64 forward.  The draft distributions are built from the ORACLE's logits."""
    shape, seed, C, M = SHAPES[key], 21, 80, 9
    ctx = gen_context_tokens(shape.vocab, C, seed)
    K, V = prefill(shape, seed, ctx)
    parents = gen_chain(M)
    T = 0.9
    # draft tokens depend on the verifier's logits at the previous node: build the chain node by node
    tokens = np.zeros(M, dtype=np.int32)
    tokens[0] = 17
    p_draft = np.zeros((M - 1, shape.vocab), dtype=np.float32)
    for i in range(M - 1):
        case = Case(shape, seed, [K], [V], tokens, parents, C + tree_depths(parents))
        lg = case.run_oracle()[0]["logits"]
        pd, tk = gen_draft_distributions(lg[: i + 2], T, seed + i, noise=0.5)
        p_draft[i], tokens[i + 1] = pd[i], tk[i + 1]
    case = Case(shape, seed, [K], [V], tokens, parents, C + tree_depths(parents))
    want_logits = case.run_oracle()[0]["logits"][None]
    gpu = case.run_gpu(0.0, CRIT_MARGIN)
    logits_dev = gpu["_ver"].logits.reshape(1, M, shape.vocab).contiguous()
    dev = lambda x, dt: torch.from_numpy(np.ascontiguousarray(x)).to(dt).cuda()
    stats = np.zeros(3, dtype=int)
    for s in range(12):
        ua, us = gen_uniforms(seed + s, 1, M)
        for lam, resample in [(0.0, RESAMPLE_RESIDUAL), (0.15, RESAMPLE_DIRECT)]:
            out = sample_decide(logits_dev, dev(tokens[None], torch.int32), dev(p_draft[None], torch.float32),
                                dev(ua, torch.float32), dev(us, torch.float32), T, lam, CRIT_MARGIN, 1, resample)
            torch.cuda.synchronize()
            got = {k: v.cpu().numpy() for k, v in out.items() if not k.startswith("_")}
            stats += compare(want_logits, tokens[None], p_draft[None], ua, us, T, lam, CRIT_MARGIN, 1, resample, got,
                             eps=tol, tol_stat=tol)
    assert stats[0] >= 16, stats
