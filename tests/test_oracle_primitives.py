"""Pins for the oracle's primitives: each is checked against a closed form, a textbook
identity or a library routine, none against the oracle's own formula."""
import numpy as np
import pytest
import torch

from oracle import apply_rope, bf16_round, rmsnorm, rope_angles, node_stats


def test_bf16_round_matches_library_conversion():
    g = np.random.default_rng(0)
    x = (g.standard_normal(200000) * np.exp(g.uniform(-20, 20, 200000))).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy().astype(np.float64)
    got = bf16_round(x.astype(np.float64))
    assert np.array_equal(got, want)


def test_bf16_round_ties_to_even_and_exact_values():
    # 1 + 2^-8 is halfway between 1 and 1 + 2^-7: ties to even mantissa -> 1.0
    assert bf16_round(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    # 1 + 3*2^-8 is halfway between 1+2^-7 and 1+2^-6 -> even is 1+2^-6
    assert bf16_round(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    # single rounding straight from fp64: just above the tie goes up even though a
    # float32 intermediate would have landed exactly on the tie
    assert bf16_round(np.array([1.0 + 2.0 ** -8 + 2.0 ** -40]))[0] == 1.0 + 2.0 ** -7
    v = np.array([0.0, -0.0, 0.5, -3.0, 2.0 ** -100, 1.5 * 2.0 ** 100])
    assert np.array_equal(bf16_round(v), v)


def test_rmsnorm_closed_forms():
    H = 64
    x = np.full((1, H), 3.0)
    w = np.arange(1, H + 1, dtype=np.float64)
    # constant row: x / sqrt(9 + eps) * w
    assert np.allclose(rmsnorm(x, w, 0.0), w, rtol=0, atol=1e-15)
    assert np.allclose(rmsnorm(x, w, 7.0), 3.0 / 4.0 * w, rtol=0, atol=1e-15)
    # one-hot row: mean square = a^2/H
    e = np.zeros((1, H)); e[0, 5] = -2.0
    out = rmsnorm(e, np.ones(H), 0.0)
    assert out[0, 5] == pytest.approx(-np.sqrt(H)) and np.count_nonzero(out) == 1
    # library routine
    g = np.random.default_rng(1)
    x = g.standard_normal((5, H)); w = g.standard_normal(H)
    want = torch.nn.functional.rms_norm(torch.from_numpy(x), (H,), torch.from_numpy(w), 1e-6).numpy()
    assert np.allclose(rmsnorm(x, w, 1e-6), want, rtol=1e-13, atol=1e-13)


def test_rope_is_complex_rotation_of_half_split_pairs():
    g = np.random.default_rng(2)
    d, T, heads, base = 16, 7, 3, 1e4
    t = g.standard_normal((T, heads, d))
    pos = np.array([0, 1, 2, 5, 100, 1000, 4099])
    ang = rope_angles(pos, d, base)
    # closed form of the angles
    for j in range(d // 2):
        assert np.allclose(ang[:, j], pos * base ** (-2.0 * j / d), rtol=1e-14)
    out = apply_rope(t, ang)
    z = (t[..., : d // 2] + 1j * t[..., d // 2:]) * np.exp(1j * ang)[:, None, :]
    assert np.allclose(out[..., : d // 2], z.real, atol=1e-13)
    assert np.allclose(out[..., d // 2:], z.imag, atol=1e-13)
    # position 0 is the identity; norms are preserved
    assert np.array_equal(out[0], t[0])
    assert np.allclose(np.linalg.norm(out, axis=-1), np.linalg.norm(t, axis=-1))


def test_rope_scores_depend_only_on_relative_position():
    g = np.random.default_rng(3)
    d = 32
    q = g.standard_normal((1, 1, d)); k = g.standard_normal((1, 1, d))
    def score(pq, pk):
        return float(np.sum(apply_rope(q, rope_angles([pq], d, 1e4)) * apply_rope(k, rope_angles([pk], d, 1e4))))
    assert score(10, 3) == pytest.approx(score(1010, 1003), abs=1e-10)
    assert score(10, 3) != pytest.approx(score(10, 4), abs=1e-6)


def test_node_stats_closed_forms():
    V = 50
    # all-equal logits: uniform distribution, first index wins, duplicated maximum -> margin 0
    s = node_stats(np.zeros((1, V)))
    assert s["argmax"][0] == 0 and s["conf"][0] == pytest.approx(1 / V) and s["margin"][0] == 0.0
    # two-point mass: logits (a, b, -inf...) -> sigmoid
    row = np.full((1, V), -1e9); row[0, 7] = 2.0; row[0, 3] = 0.5
    s = node_stats(row)
    p1 = 1 / (1 + np.exp(-1.5))
    assert s["argmax"][0] == 7
    assert s["conf"][0] == pytest.approx(p1, rel=1e-12)
    assert s["top2"][0] == pytest.approx(1 - p1, rel=1e-12)
    assert s["margin"][0] == pytest.approx(2 * p1 - 1, rel=1e-12)
    # tie between two maxima: lowest index, margin 0
    row = np.zeros((1, V)); row[0, 9] = row[0, 4] = 3.0
    s = node_stats(row)
    assert s["argmax"][0] == 4 and s["margin"][0] == 0.0 and s["l1"][0] == s["l2"][0]
    # library softmax / topk on random rows; bounds
    g = np.random.default_rng(4)
    L = g.standard_normal((6, 300)) * 4
    s = node_stats(L)
    p = torch.softmax(torch.from_numpy(L), dim=-1)
    top = torch.topk(p, 2, dim=-1)
    assert np.array_equal(s["argmax"], top.indices[:, 0].numpy())
    assert np.allclose(s["conf"], top.values[:, 0].numpy(), rtol=1e-12)
    assert np.allclose(s["top2"], top.values[:, 1].numpy(), rtol=1e-12)
    assert np.all(s["conf"] >= 1 / 300) and np.all(s["conf"] <= 1) and np.all(s["margin"] >= 0)
    assert np.all(s["margin"] <= s["conf"])
