"""Oracle for the sampling (temperature > 0) form of the verification decision on a
draft CHAIN.  Test infrastructure, not the product.

Paper Sec. 2.1: each draft token x_i is accepted with probability
min(1, p_v,i(x_i) / p_d,i(x_i)); at the first rejection everything to its right is
dropped and the replacement is drawn from norm(max(0, p_v,i - p_d,i)).  Sec. 3.2 Eq. 6
states the same Bernoulli variable s_i for the proxy; Eq. 7 - Eq. 9 and the routing
(Case I / Case II) are unchanged.  Algorithm 1 writes the token after the accepted
prefix as a plain draw from the verifier's distribution at that position; both forms
are here (`RESAMPLE_RESIDUAL`, the lossless rule of Sec. 2.1, and `RESAMPLE_DIRECT`,
Algorithm 1 as printed).  When every draft token is accepted there is no draft
distribution at the next position and both forms draw from p_v,k+1.

All randomness comes in as arguments: u_accept[i] in [0, 1) decides s_i, u_sample in
[0, 1) drives one inverse-CDF draw.  Distributions are softmax(logits / T) in fp64; the
trust predicate g (Eq. 8) is evaluated on that same tempered distribution.

Indexing as in the greedy oracle: the distribution the paper calls p_{j+1} is emitted AT
chain node j (node 0 = last committed token, node j = j-th draft token), and
p_draft[j] is the drafter's distribution from which node j+1's token was drawn.
"""
from __future__ import annotations

from typing import Dict

import numpy as np

from .decision import CRIT_MARGIN

RESAMPLE_RESIDUAL = 0  # Sec. 2.1: norm(max(0, p_v - p_d)) at the first rejection
RESAMPLE_DIRECT = 1    # Algorithm 1 as printed: draw from p_v at that position


def tempered_softmax(logits: np.ndarray, temperature: float) -> np.ndarray:
    z = np.asarray(logits, dtype=np.float64) / float(temperature)
    e = np.exp(z - z.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def accept_probability(p_v: np.ndarray, p_d: np.ndarray, x: int) -> float:
    """min(1, p_v(x) / p_d(x)) (Eq. 6).  A token the drafter gives probability 0 cannot have
    been drawn from it; the ratio is then taken as 1 if p_v(x) > 0, else 0."""
    if p_d[x] <= 0.0:
        return 1.0 if p_v[x] > 0.0 else 0.0
    return float(min(1.0, p_v[x] / p_d[x]))


def residual_mass(p_v: np.ndarray, p_d: np.ndarray) -> np.ndarray:
    """max(0, p_v - p_d), not normalised."""
    return np.maximum(0.0, np.asarray(p_v, dtype=np.float64) - np.asarray(p_d, dtype=np.float64))


def residual_distribution(p_v: np.ndarray, p_d: np.ndarray) -> np.ndarray:
    r = residual_mass(p_v, p_d)
    return r / r.sum()


def inverse_cdf(mass: np.ndarray, u: float) -> int:
    """Smallest v with mass[0] + ... + mass[v] > u * sum(mass): token v owns the half-open
    interval [cdf(v-1), cdf(v)) of the unit interval scaled by the total."""
    c = np.cumsum(np.asarray(mass, dtype=np.float64))
    v = int(np.searchsorted(c, u * c[-1], side="right"))
    return min(v, len(c) - 1)


def sample_decide(logits: np.ndarray, tokens: np.ndarray, p_draft: np.ndarray, u_accept: np.ndarray,
                  u_sample: float, temperature: float, lam: float, criterion: int = CRIT_MARGIN,
                  n_forced: int = 1, resample: int = RESAMPLE_RESIDUAL) -> Dict[str, object]:
    """One sequence.  logits [M, V] of chain nodes 0..M-1, tokens [M], p_draft [M-1, V],
    u_accept [M] (entry i decides draft node i; entries below n_forced are unused).

    Walk from node n_forced-1: test g at the current node first (tau_a = tau_m is Case II,
    as in the greedy rule), then s of the next draft token.  Returns accepted_len,
    token (-1 in Case II), escalate, path, and for the tests: `row` the node whose
    distribution yielded the token (-1 if none), `mass` the unnormalised distribution it was
    drawn from, and `slack` = min over tested nodes of |u * p_d(x) - p_v(x)| / p_v(x)."""
    logits = np.asarray(logits, dtype=np.float64)
    M = logits.shape[0]
    p = tempered_softmax(logits, temperature)
    cur, acc, token, esc, row, mass = n_forced - 1, 0, -1, 0, -1, None
    path, slack = [cur], np.inf
    while True:
        srt = np.sort(p[cur])
        conf, second = srt[-1], (srt[-2] if srt.size > 1 else 0.0)
        stat = conf - second if criterion == CRIT_MARGIN else conf
        if not stat >= lam:
            esc = 1
            break
        if cur + 1 >= M:            # every draft token accepted: bonus from p_{k+1}
            row, mass = cur, p[cur]
            break
        x = int(tokens[cur + 1])
        q = float(p_draft[cur][x])
        u = float(u_accept[cur + 1])
        slack = min(slack, abs(u * q - p[cur][x]) / max(p[cur][x], 1e-300))
        if u < accept_probability(p[cur], p_draft[cur], x):
            cur += 1
            acc += 1
            path.append(cur)
            continue
        row = cur
        mass = residual_mass(p[cur], p_draft[cur]) if resample == RESAMPLE_RESIDUAL else p[cur]
        break
    if mass is not None:
        token = inverse_cdf(mass, u_sample)
    return {"accepted_len": acc, "token": token, "escalate": esc, "path": path, "row": row,
            "mass": mass, "slack": slack}
