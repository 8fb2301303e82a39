"""Oracle: committing a verified path to the cache and running several rounds.  Test infrastructure.

Standard speculative decoding (paper Sec. 2.1; Alg. 1 in the appendix) appends, after every
round, the accepted draft prefix and one more token from the verifier (the correction at the
first mismatch, or the bonus token after a fully accepted draft) to the output sequence.  In
cache terms: the root of the round (the last emitted token, whose keys / values were not cached
yet) and the accepted drafts become context; the extra token is the next round's root.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Sequence, Tuple

import numpy as np

from .decision import CRIT_MARGIN, decide, node_stats
from .forward import OracleWeights, causal_forward, verify_forward


def commit(k_ctx: np.ndarray, v_ctx: np.ndarray, k_new: np.ndarray, v_new: np.ndarray,
           nodes: Sequence[int]) -> Tuple[np.ndarray, np.ndarray]:
    """Cache after a round.  k_ctx, v_ctx: [L, n_kv, C, d]; k_new, v_new: [L, n_kv, M, d] as the
    verification pass appends them (rounded to the storage type); nodes: the root and the
    approved drafts in path order.  Returns caches of length C + len(nodes)."""
    idx = np.asarray(list(nodes), dtype=np.int64)
    return (np.concatenate([k_ctx, k_new[:, :, idx, :]], axis=2),
            np.concatenate([v_ctx, v_new[:, :, idx, :]], axis=2))


def greedy_decode(W: OracleWeights, shape, prompt: Sequence[int], n_new: int) -> List[int]:
    """Plain autoregressive greedy decoding, no cache: the textbook definition the rounds are
    pinned to.  (For bf16 storage every earlier token counts as cached when the next is computed.)"""
    seq = [int(t) for t in prompt]
    for _ in range(n_new):
        lg = causal_forward(W, shape, seq, last_only=True, n_cached=len(seq) - 1)["logits"][0]
        seq.append(int(np.argmax(lg)))
    return seq


def verify_rounds(W: OracleWeights, shape, prompt: Sequence[int],
                  draft_fn: Callable[[int, List[int]], Tuple[np.ndarray, np.ndarray]],
                  n_rounds: int, lam: float = 0.0, criterion: int = CRIT_MARGIN) -> Dict[str, list]:
    """Rounds of draft -> verify -> commit with ONE verifier.

    draft_fn(round, sequence so far) -> (parents [M], tokens [M]); tokens[0] is overwritten with
    the round's root (the last emitted token).  With lam = 0 the margin test never fires and every
    round is standard greedy acceptance, so the emitted sequence equals greedy_decode's.
    If a round escalates (lam > 0) the loop stops there: what follows needs the target.
    Returns the sequence, and per round the decision and the cache length before it."""
    seq = [int(t) for t in prompt]
    pre = causal_forward(W, shape, seq[:-1]) if len(seq) > 1 else None
    L, nkv, d = shape.n_layers, shape.n_kv_heads, shape.head_dim
    k_ctx = pre["K"] if pre is not None else np.zeros((L, nkv, 0, d))
    v_ctx = pre["V"] if pre is not None else np.zeros((L, nkv, 0, d))
    rounds = []
    for r in range(n_rounds):
        parents, tokens = draft_fn(r, seq)
        parents = np.asarray(parents, dtype=np.int32)
        tokens = np.asarray(tokens, dtype=np.int32).copy()
        tokens[0] = seq[-1]
        depth = np.zeros(len(parents), dtype=np.int64)
        for i in range(1, len(parents)):
            depth[i] = depth[parents[i]] + 1
        C = k_ctx.shape[2]
        out = verify_forward(W, shape, k_ctx, v_ctx, tokens, parents, C + depth)
        st = node_stats(out["logits"])
        dec = decide(tokens, parents, st["argmax"], st["conf"], st["margin"], lam, criterion, 1)
        rounds.append({"ctx_len": C, "tokens": tokens, "parents": parents, "decision": dec, "stats": st})
        path = [int(v) for v in dec["path"]]
        k_ctx, v_ctx = commit(k_ctx, v_ctx, out["k_new"], out["v_new"], path)
        seq += [int(tokens[i]) for i in path[1:]]
        if dec["escalate"]:
            break
        seq.append(int(dec["token"]))
    return {"sequence": seq, "rounds": rounds, "k_ctx": k_ctx, "v_ctx": v_ctx}


def trispec_rounds(Wp: OracleWeights, shape_p, Wt: OracleWeights, shape_t, prompt: Sequence[int],
                   draft_fn: Callable[[int, List[int]], Tuple[np.ndarray, np.ndarray]], n_rounds: int,
                   lam: float, criterion: int = CRIT_MARGIN, max_nodes: int = 64) -> Dict[str, list]:
    """Rounds of the ternary scheme (Alg. 1, greedy): draft -> proxy pre-verification ->
    Case I (tau_a < tau_m: the proxy's own correction / bonus token ends the round) or
    Case II (tau_a >= tau_m: the target re-verifies what the proxy did not vouch for, Eq. 10).

    Each model keeps its own cache.  The proxy sees every token.  The target only runs in
    Case II, so its cache lags: the committed tokens it has not seen yet are prepended to its
    input as part of the forced chain (they are certain, the pass only has to produce their
    keys / values), followed by the proxy-approved path v_0..v_tau_m and the subtree under
    v_tau_m.  If that exceeds max_nodes, the unseen tokens go in by plain catch-up passes
    first.  Returns the emitted sequence and one record per round."""
    from .decision import prune_reroot

    seq = [int(t) for t in prompt]

    def prefill(W, shape):
        if len(seq) > 1:
            o = causal_forward(W, shape, seq[:-1])
            return o["K"], o["V"]
        z = np.zeros((shape.n_layers, shape.n_kv_heads, 0, shape.head_dim))
        return z, z.copy()

    kp, vp = prefill(Wp, shape_p)
    kt, vt = prefill(Wt, shape_t)
    records = []
    for r in range(n_rounds):
        parents, tokens = draft_fn(r, seq)
        parents = np.asarray(parents, dtype=np.int32)
        tokens = np.asarray(tokens, dtype=np.int32).copy()
        tokens[0] = seq[-1]
        depth = np.zeros(len(parents), dtype=np.int64)
        for i in range(1, len(parents)):
            depth[i] = depth[parents[i]] + 1
        Cp = kp.shape[2]
        positions = Cp + depth
        out = verify_forward(Wp, shape_p, kp, vp, tokens, parents, positions)
        st = node_stats(out["logits"])
        dec = decide(tokens, parents, st["argmax"], st["conf"], st["margin"], lam, criterion, 1)
        path = [int(v) for v in dec["path"]]
        rec = {"proxy": dec, "proxy_stats": st, "escalate": int(dec["escalate"]), "catch_up": 0}
        if not dec["escalate"]:                                   # Case I
            kp, vp = commit(kp, vp, out["k_new"], out["v_new"], path)
            seq += [int(tokens[i]) for i in path[1:]] + [int(dec["token"])]
            records.append(rec)
            continue
        # Case II
        pr = prune_reroot(tokens, parents, positions, path)
        t_len = kt.shape[2]
        unseen = seq[t_len:-1]                                     # committed, not yet cached by the target
        fits = len(unseen) + len(pr["tokens"]) <= max_nodes
        while unseen and not fits:                                 # plain catch-up passes over all of them
            take = min(len(unseen), max_nodes)
            chunk = np.asarray(unseen[:take], dtype=np.int32)
            o = verify_forward(Wt, shape_t, kt, vt, chunk, np.arange(-1, take - 1), t_len + np.arange(take))
            kt, vt = commit(kt, vt, o["k_new"], o["v_new"], list(range(take)))
            t_len += take
            unseen = unseen[take:]
            rec["catch_up"] += 1
        u = len(unseen)
        tok_t = np.concatenate([np.asarray(unseen, dtype=np.int32), pr["tokens"]])
        par_t = np.concatenate([np.arange(-1, u - 1, dtype=np.int32),
                                np.where(pr["parents"] < 0, u - 1, pr["parents"] + u).astype(np.int32)])
        pos_t = np.concatenate([t_len + np.arange(u), pr["positions"]])
        n_forced_t = u + pr["n_forced"]
        out_t = verify_forward(Wt, shape_t, kt, vt, tok_t, par_t, pos_t)
        st_t = node_stats(out_t["logits"])
        dec_t = decide(tok_t, par_t, st_t["argmax"], st_t["conf"], st_t["margin"], 0.0, CRIT_MARGIN, n_forced_t)
        path_t = [int(v) for v in dec_t["path"]]                  # starts at v_tau_m (node n_forced_t - 1)
        kt, vt = commit(kt, vt, out_t["k_new"], out_t["v_new"], list(range(n_forced_t - 1)) + path_t)
        extra = [int(pr["old_id"][n - u]) for n in path_t[1:]]    # the drafts the target accepted, old ids
        kp, vp = commit(kp, vp, out["k_new"], out["v_new"], path + extra)
        seq += [int(tokens[i]) for i in path[1:] + extra] + [int(dec_t["token"])]
        rec.update({"target": dec_t, "target_stats": st_t, "target_nodes": len(tok_t), "n_forced_t": n_forced_t})
        records.append(rec)
    return {"sequence": seq, "rounds": records, "kp": kp, "vp": vp, "kt": kt, "vt": vt}


def trispec_sample_rounds(Wp: OracleWeights, shape_p, Wt: OracleWeights, shape_t, prompt: Sequence[int],
                          draft_fn: Callable[[int, List[int], np.ndarray], Dict[str, np.ndarray]], n_rounds: int,
                          lam: float, temperature: float, criterion: int = CRIT_MARGIN, resample: int = 0,
                          max_nodes: int = 64) -> Dict[str, list]:
    """Rounds of the ternary scheme at temperature > 0 on draft CHAINS — Alg. 1 as printed: the
    drafter samples x_1..x_k, the proxy accepts each with probability min(1, p_p / p_d) (Eq. 6),
    the margin rule gives tau_m (Eq. 8, 9), and either the proxy ends the round (tau_a < tau_m) or
    the target verifies the whole chain with x_1..x_tau_m taken as approved and ends it.

    draft_fn(round, sequence so far, proxy cache length) -> dict with
      tokens [k+1] (entry 0 is overwritten with the round's root), p_draft [k, V],
      u_accept_p [k+1], u_sample_p, u_accept_t [k+1], u_sample_t      (uniforms in [0, 1)).
    The drafter is an input: whatever distributions it reports are the p_d of Eq. 6.
    Caches, lag of the target and catch-up passes as in trispec_rounds."""
    from .sampling import sample_decide

    seq = [int(t) for t in prompt]

    def prefill(W, shape):
        if len(seq) > 1:
            o = causal_forward(W, shape, seq[:-1])
            return o["K"], o["V"]
        z = np.zeros((shape.n_layers, shape.n_kv_heads, 0, shape.head_dim))
        return z, z.copy()

    kp, vp = prefill(Wp, shape_p)
    kt, vt = prefill(Wt, shape_t)
    records = []
    for r in range(n_rounds):
        d = draft_fn(r, seq, kp.shape[2])
        tokens = np.asarray(d["tokens"], dtype=np.int32).copy()
        tokens[0] = seq[-1]
        M = len(tokens)
        p_draft = np.asarray(d["p_draft"], dtype=np.float64)
        chain = np.arange(-1, M - 1)
        Cp = kp.shape[2]
        out = verify_forward(Wp, shape_p, kp, vp, tokens, chain, Cp + np.arange(M))
        dec = sample_decide(out["logits"], tokens, p_draft, d["u_accept_p"], float(d["u_sample_p"]), temperature,
                            lam, criterion, 1, resample)
        path = list(dec["path"])
        rec = {"proxy": dec, "proxy_logits": out["logits"], "escalate": int(dec["escalate"]), "catch_up": 0,
               "tokens": tokens}
        if not dec["escalate"]:                                   # Case I
            kp, vp = commit(kp, vp, out["k_new"], out["v_new"], path)
            seq += [int(tokens[i]) for i in path[1:]] + [int(dec["token"])]
            records.append(rec)
            continue
        # Case II: the whole chain goes to the target, nodes 0..tau_m forced
        tau_m = dec["accepted_len"]
        t_len = kt.shape[2]
        unseen = seq[t_len:-1]
        fits = len(unseen) + M <= max_nodes
        while unseen and not fits:
            take = min(len(unseen), max_nodes)
            chunk = np.asarray(unseen[:take], dtype=np.int32)
            o = verify_forward(Wt, shape_t, kt, vt, chunk, np.arange(-1, take - 1), t_len + np.arange(take))
            kt, vt = commit(kt, vt, o["k_new"], o["v_new"], list(range(take)))
            t_len += take
            unseen = unseen[take:]
            rec["catch_up"] += 1
        u = len(unseen)
        tok_t = np.concatenate([np.asarray(unseen, dtype=np.int32), tokens])
        n_t = u + M
        pd_t = np.zeros((n_t - 1, p_draft.shape[1]))
        pd_t[u:] = p_draft                                         # row u + i judges node u + i + 1 = draft i + 1
        ua_t = np.zeros(n_t)
        ua_t[u:] = d["u_accept_t"]
        n_forced_t = u + tau_m + 1
        out_t = verify_forward(Wt, shape_t, kt, vt, tok_t, np.arange(-1, n_t - 1), t_len + np.arange(n_t))
        dec_t = sample_decide(out_t["logits"], tok_t, pd_t, ua_t, float(d["u_sample_t"]), temperature, 0.0,
                              CRIT_MARGIN, n_forced_t, resample)
        path_t = list(dec_t["path"])                              # starts at node n_forced_t - 1
        kt, vt = commit(kt, vt, out_t["k_new"], out_t["v_new"], list(range(n_forced_t - 1)) + path_t)
        extra = [n - u for n in path_t[1:]]                       # drafts the target accepted, chain ids
        kp, vp = commit(kp, vp, out["k_new"], out["v_new"], path + extra)
        seq += [int(tokens[i]) for i in path[1:] + extra] + [int(dec_t["token"])]
        rec.update({"target": dec_t, "target_logits": out_t["logits"], "target_nodes": n_t,
                    "n_forced_t": n_forced_t, "u": u})
        records.append(rec)
    return {"sequence": seq, "rounds": records, "kp": kp, "vp": vp, "kt": kt, "vt": vt}
