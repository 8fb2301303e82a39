"""Oracle for the per-node statistics and the ternary routing decision.
Test infrastructure, not the product.

Paper Sec. 3.2: greedy acceptance s_i = 1{x_p,i = x_d,i} and tau_a (Eq. 6
greedy form, Eq. 7); margin predicate g and trusted prefix tau_m (Eq. 8,
Eq. 9); routing Case I (tau_a < tau_m: keep x_1..x_tau_a and the proxy's own
token for position tau_a+1) and Case II (tau_a >= tau_m: keep x_1..x_tau_m and
hand the rest to the target).  "Routing Criteria" (Sec. 4.3) also evaluates
the plain top-1 probability and an entropy criterion in place of the margin; the
entropy criterion is only cited there ("composite"), not defined, so what is built
is the plain Shannon entropy of the verifier's distribution, trusted when it is AT
MOST the threshold (a reading, recorded as such).  The appendix on relaxed
verification accepts a draft token that lies within the verifier's top-k
candidates; `draft_ranks` gives the rank that rule needs and `decide(top_k=...)`
the walk under it.

Indexing.  The distribution the paper calls p_{j+1} is the one the verifier
emits AT path node v_j (v_0 = the root = last committed token, v_j = j-th
accepted draft token).
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

import numpy as np

CRIT_MARGIN = 0  # g = 1{top1 - top2 >= lambda}   (Eq. 8, the paper's default)
CRIT_TOP1 = 1    # g = 1{top1 >= lambda}          (Sec. 4.3 alternative)
CRIT_ENTROPY = 2  # g = 1{H(p) <= lambda}, H in nats (Sec. 4.3 names an entropy criterion; this reading is ours)


def node_stats(logits: np.ndarray) -> Dict[str, np.ndarray]:
    """Per node: argmax token (lowest index among equal maxima), top-1 and top-2
    softmax probabilities (temperature 1), their margin, the two largest logits, and the
    Shannon entropy -sum p ln p of the distribution (0 ln 0 = 0).
    top-2 is the second-largest ENTRY of p, so a duplicated maximum gives margin 0."""
    logits = np.asarray(logits, dtype=np.float64)
    M = logits.shape[0]
    arg = np.empty(M, dtype=np.int32)
    conf = np.empty(M)
    top2 = np.empty(M)
    l1 = np.empty(M)
    l2 = np.empty(M)
    ent = np.empty(M)
    for i in range(M):
        row = logits[i]
        p = np.exp(row - row.max())
        p /= p.sum()
        nz = p > 0
        ent[i] = -np.sum(p[nz] * np.log(p[nz]))
        a = int(np.argmax(row))  # first occurrence
        rest = np.delete(p, a)
        arg[i] = a
        conf[i] = p[a]
        top2[i] = rest.max() if rest.size else 0.0
        l1[i] = row[a]
        l2[i] = np.delete(row, a).max() if rest.size else -np.inf
    return {"argmax": arg, "conf": conf, "top2": top2, "margin": conf - top2,
            "l1": l1, "l2": l2, "entropy": ent}


def draft_ranks(logits: np.ndarray, tokens: Sequence[int], parents: Sequence[int]) -> np.ndarray:
    """rank[i] of draft node i > 0: how many vocabulary entries the verifier puts before node i's
    token in the distribution emitted at its PARENT (larger logit, or equal logit and lower token
    id); 0 means the token is the parent's argmax, rank < k that it is among the top-k candidates
    (the relaxed verification of the appendix).  rank[0] = -1 (the root was not drafted)."""
    logits = np.asarray(logits, dtype=np.float64)
    out = np.full(len(tokens), -1, dtype=np.int64)
    for i in range(1, len(tokens)):
        row, x = logits[parents[i]], int(tokens[i])
        out[i] = int(np.sum(row > row[x]) + np.sum(row[:x] == row[x]))
    return out


def _trusted(conf: float, margin: float, lam: float, criterion: int, entropy: float = None) -> bool:
    if criterion == CRIT_ENTROPY:
        return bool(entropy <= lam)
    v = margin if criterion == CRIT_MARGIN else conf
    return bool(v >= lam)


def decide(tokens: Sequence[int], parents: Sequence[int], argmax: Sequence[int],
           conf: Sequence[float], margin: Sequence[float], lam: float,
           criterion: int = CRIT_MARGIN, n_forced: int = 1, entropy: Sequence[float] = None,
           ranks: Sequence[int] = None, top_k: int = 1) -> Dict[str, object]:
    """Greedy walk down the draft tree = tree form of Eq. 7 / Eq. 9 + routing.

    Start at node n_forced-1 (the last already-committed node).  At the current
    node v_j: if g(p_{j+1}) = 0 the trusted prefix ends here (tau_m = j <= tau_a,
    Case II): escalate.  Otherwise follow the child whose draft token equals the
    verifier's argmax; with no such child the first rejection is here
    (tau_a = j < tau_m, Case I) and the argmax is the correction / bonus token.
    The margin test comes first because tau_a = tau_m is Case II.
    criterion CRIT_ENTROPY needs `entropy` (per node).  top_k > 1 is the relaxed acceptance of
    the appendix: a child is followed if its token is among the verifier's top_k candidates
    (ranks[child] < top_k, `draft_ranks`), the lowest-numbered such child first; where the walk
    stops without escalating, the verifier's own token is still its argmax.
    """
    n = len(tokens)
    children: List[List[int]] = [[] for _ in range(n)]
    for i in range(1, n):
        children[parents[i]].append(i)
    cur = n_forced - 1
    acc = 0
    path = [cur]
    while True:
        if not _trusted(conf[cur], margin[cur], lam, criterion, None if entropy is None else entropy[cur]):
            return {"accepted_len": acc, "token": -1, "escalate": 1, "path": path}
        t = int(argmax[cur])
        nxt = -1
        for c in children[cur]:  # ascending node index: lowest matching child wins
            if (int(tokens[c]) == t) if top_k <= 1 else (0 <= int(ranks[c]) < top_k):
                nxt = c
                break
        if nxt < 0:
            return {"accepted_len": acc, "token": t, "escalate": 0, "path": path}
        cur = nxt
        acc += 1
        path.append(cur)


# -- the chain definitions exactly as printed (used to pin `decide`) ---------


def chain_tau_a(s: Sequence[int]) -> int:
    """Eq. 7.  s = (s_1..s_k); tau_a = min({i | 0 <= i <= k-1, s_{i+1} = 0} U {k})."""
    k = len(s)
    return min([i for i in range(0, k) if s[i] == 0] + [k])


def chain_tau_m(g: Sequence[int]) -> int:
    """Eq. 9.  g = (g(p_1)..g(p_{k+1})); tau_m = min({i | 0 <= i <= k, g(p_{i+1}) = 0} U {k+1})."""
    k = len(g) - 1
    return min([i for i in range(0, k + 1) if g[i] == 0] + [k + 1])


def chain_round_output(s: Sequence[int], g: Sequence[int]) -> Tuple[int, int, int]:
    """Routing of Sec. 3.2 on a chain: returns (case, accepted_len, index of the
    distribution that supplies the extra token or 0).  Case I: accept tau_a drafts and
    take the proxy token of position tau_a+1.  Case II: accept tau_m drafts, escalate."""
    ta, tm = chain_tau_a(s), chain_tau_m(g)
    if ta < tm:
        return (1, ta, ta + 1)
    return (2, tm, 0)


# -- tie flags (which nodes may legitimately flip between implementations) ---


def tie_flags(stats: Dict[str, np.ndarray], lam: float, criterion: int,
              tol: float = 1e-3) -> np.ndarray:
    """A node is tie-flagged if its routing statistic is within tol of the threshold
    or its two largest logits are within tol of each other."""
    v = stats["entropy"] if criterion == CRIT_ENTROPY else (stats["margin"] if criterion == CRIT_MARGIN else stats["conf"])
    return (np.abs(v - lam) < tol) | ((stats["l1"] - stats["l2"]) < tol)


# -- Case II: prune the accepted prefix and re-root (Sec. 3.2 (ii), Eq. 10) --


def prune_reroot(tokens: Sequence[int], parents: Sequence[int], positions: Sequence[int],
                 path: Sequence[int]) -> Dict[str, np.ndarray]:
    """Target-pass input after the proxy approved path = [v_0..v_tau_m].

    The target has no KV for the approved tokens yet, so they stay in the input as a
    forced chain (n_forced = tau_m + 1); of the draft tree only the subtree below
    v_tau_m survives (Eq. 10 conditions on x_1..x_tau_m and verifies the rest);
    every other branch is dropped.  Returns new tokens / parents / positions, the
    old node id of every kept node, and n_forced.
    """
    n = len(tokens)
    path = list(path)
    last = path[-1]
    keep = list(path)
    in_sub = [False] * n
    in_sub[last] = True
    for i in range(last + 1, n):  # parents[i] < i, so one ascending sweep finds the subtree
        if in_sub[parents[i]]:
            in_sub[i] = True
            keep.append(i)
    new_id = {old: new for new, old in enumerate(keep)}
    new_par = np.array([-1 if j == 0 else new_id[parents[old]] for j, old in enumerate(keep)],
                       dtype=np.int32)
    return {"tokens": np.asarray(tokens, dtype=np.int32)[keep],
            "parents": new_par,
            "positions": np.asarray(positions, dtype=np.int32)[keep],
            "old_id": np.asarray(keep, dtype=np.int32),
            "n_forced": len(path)}
