"""Round driver of the ternary scheme on top of the C ABI (Alg. 1 of the paper; greedy on draft
trees, and the sampling form on draft chains).

Host control flow only — a few dozen integers per round; every model pass is one
trispec_verify call and every cache update one trispec_kv_commit call.  One sequence (batch 1).

  round:  draft tree -> proxy pass (threshold lambda)
          Case I  (no escalation): commit the approved path to the proxy cache; the proxy's
                  correction / bonus token is the next root.  The target is not run.
          Case II (escalation): the target verifies [tokens it has not cached yet] + [approved
                  path v_0..v_tau_m] as a forced chain, plus the subtree under v_tau_m
                  (Eq. 10), with lambda = 0; both caches commit what was accepted; the target's
                  token is the next root.
The target's cache lags behind while rounds end at the proxy; tokens it has not seen ride along
as the head of the forced chain, or go in by plain catch-up passes when they do not fit.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np
import torch

from .binding import (CRIT_MARGIN, MAX_NODES, RESAMPLE_RESIDUAL, KVCache, Model, SampleDecider, TriSpecError, Verifier,
                      prune_reroot)


def _depths(parents: Sequence[int]) -> np.ndarray:
    d = np.zeros(len(parents), dtype=np.int32)
    for i in range(1, len(parents)):
        d[i] = d[parents[i]] + 1
    return d


class TernaryDecoder:
    def __init__(self, proxy: Model, target: Model, capacity: int, criterion: int = CRIT_MARGIN,
                 max_nodes: int = MAX_NODES):
        self.proxy, self.target = proxy, target
        self.kv_p, self.kv_t = KVCache(proxy, 1, capacity), KVCache(target, 1, capacity)
        self.criterion, self.max_nodes = criterion, max_nodes
        self._ver: Dict[tuple, Verifier] = {}
        self._dec: Dict[tuple, SampleDecider] = {}
        self.seq: List[int] = []
        self.target_passes = 0          # passes of the target that verified drafts (not catch-up)

    # -- one pass --------------------------------------------------------------------------
    def _pass(self, which: str, tokens, parents, positions, lam: float, criterion: int, n_forced: int):
        model, kv = (self.proxy, self.kv_p) if which == "p" else (self.target, self.kv_t)
        n = len(tokens)
        ver = self._ver.get((which, n))
        if ver is None:
            ver = self._ver[(which, n)] = Verifier(model, 1, n)
        tok = torch.tensor([list(map(int, tokens))], dtype=torch.int32, device="cuda")
        pos = torch.tensor([list(map(int, positions))], dtype=torch.int32, device="cuda")
        par = np.asarray([list(map(int, parents))], dtype=np.int32)
        out = ver.verify(kv, tok, par, pos, lam, criterion, n_forced, want_logits=False)
        torch.cuda.synchronize()
        return {"accepted_len": int(out["accepted_len"][0]), "token": int(out["token"][0]),
                "escalate": int(out["escalate"][0]),
                "path": [int(v) for v in out["path"][0].cpu().numpy() if v >= 0]}

    def _ingest(self, which: str, tokens: Sequence[int]) -> None:
        """Plain passes over certain tokens: a forced chain, everything committed."""
        kv = self.kv_p if which == "p" else self.kv_t
        tokens = list(tokens)
        while tokens:
            chunk, tokens = tokens[: self.max_nodes], tokens[self.max_nodes:]
            n, c = len(chunk), kv.ctx_len[0]
            self._pass(which, chunk, range(-1, n - 1), range(c, c + n), 0.0, CRIT_MARGIN, n)
            kv.commit([list(range(n))])

    # -- API -------------------------------------------------------------------------------
    def start(self, prompt: Sequence[int]) -> None:
        """Caches of both models over the prompt but its last token (the first root)."""
        self.seq = [int(t) for t in prompt]
        self.kv_p.set_len([0]); self.kv_t.set_len([0])
        self._ingest("p", self.seq[:-1])
        self._ingest("t", self.seq[:-1])

    def round(self, parents: Sequence[int], tokens: Sequence[int], lam: float) -> Dict[str, object]:
        """One round on a draft tree (tokens[0] is replaced by the current root).  Returns what
        happened; self.seq has grown by the accepted drafts and one verifier token."""
        parents = [int(p) for p in parents]
        tokens = [int(t) for t in tokens]
        tokens[0] = self.seq[-1]
        cp = self.kv_p.ctx_len[0]
        positions = cp + _depths(parents)
        pr = self._pass("p", tokens, parents, positions, lam, self.criterion, 1)
        rec = {"proxy": pr, "escalate": pr["escalate"], "catch_up": 0}
        path = pr["path"]
        if not pr["escalate"]:                                               # Case I
            self.kv_p.commit([path])
            self.seq += [tokens[i] for i in path[1:]] + [pr["token"]]
            return rec
        t_len = self.kv_t.ctx_len[0]                                         # Case II
        unseen = self.seq[t_len:-1]
        sub = None
        try:       # the pruned, re-rooted tree behind the tokens the target has not cached yet (library call)
            sub = prune_reroot(tokens, parents, positions, path, unseen, t_len)
        except TriSpecError as e:
            if e.code != -3:                                                 # TRISPEC_ENODES: does not fit
                raise
        if sub is None or len(sub["tokens"]) > self.max_nodes:
            before = self.kv_t.ctx_len[0]
            self._ingest("t", unseen)
            rec["catch_up"] = (self.kv_t.ctx_len[0] - before + self.max_nodes - 1) // self.max_nodes
            sub = prune_reroot(tokens, parents, positions, path)
        tok_t, n_forced = sub["tokens"], sub["n_forced"]
        tr = self._pass("t", tok_t, sub["parents"], sub["positions"], 0.0, CRIT_MARGIN, n_forced)
        self.target_passes += 1
        self.kv_t.commit([list(range(n_forced - 1)) + tr["path"]])
        extra = [sub["old_id"][n] for n in tr["path"][1:]]                   # drafts the target accepted, old ids
        self.kv_p.commit([path + extra])
        self.seq += [tokens[i] for i in path[1:] + extra] + [tr["token"]]
        rec.update({"target": tr, "target_nodes": len(tok_t), "n_forced_t": n_forced})
        return rec

    # -- sampling form (temperature > 0), draft chains -----------------------------------------
    def _pass_sample(self, which: str, tokens, positions, p_draft, u_accept, u_sample, lam: float, criterion: int,
                     n_forced: int, temperature: float, resample: int):
        """One pass over a chain with its logits kept, then trispec_sample_decide on them."""
        model, kv = (self.proxy, self.kv_p) if which == "p" else (self.target, self.kv_t)
        n = len(tokens)
        ver = self._ver.get((which, n, "logits"))
        if ver is None:
            ver = self._ver[(which, n, "logits")] = Verifier(model, 1, n, debug_logits=True)
        dec = self._dec.get((which, n))
        if dec is None:
            dec = self._dec[(which, n)] = SampleDecider(1, n, model.cfg.vocab)
        tok = torch.tensor([list(map(int, tokens))], dtype=torch.int32, device="cuda")
        pos = torch.tensor([list(map(int, positions))], dtype=torch.int32, device="cuda")
        par = np.arange(-1, n - 1, dtype=np.int32)[None]
        ver.verify(kv, tok, par, pos, 0.0, CRIT_MARGIN, n_forced, want_logits=True)
        f32 = dict(dtype=torch.float32, device="cuda")
        pd = torch.as_tensor(np.ascontiguousarray(p_draft, dtype=np.float32)[None], **f32)
        ua = torch.as_tensor(np.ascontiguousarray(u_accept, dtype=np.float32)[None], **f32)
        us = torch.as_tensor(np.asarray([u_sample], dtype=np.float32), **f32)
        out = dec.decide(ver.logits, tok, pd, ua, us, temperature, lam, criterion, n_forced, resample)
        torch.cuda.synchronize()
        return {"accepted_len": int(out["accepted_len"][0]), "token": int(out["token"][0]),
                "escalate": int(out["escalate"][0]),
                "path": [int(v) for v in out["path"][0].cpu().numpy() if v >= 0]}

    def round_sample(self, tokens: Sequence[int], p_draft: np.ndarray, u_accept_p, u_sample_p: float, u_accept_t,
                     u_sample_t: float, lam: float, temperature: float,
                     resample: int = RESAMPLE_RESIDUAL) -> Dict[str, object]:
        """One round at temperature > 0 on a draft chain tokens[0..k] (tokens[0] is replaced by the
        current root): p_draft [k, vocab] are the drafter's distributions, the uniforms are the
        caller's.  The proxy accepts by Eq. 6 and routes by Eq. 8 / 9; on escalation the target
        verifies the whole chain with x_1..x_tau_m taken as approved."""
        tokens = [int(t) for t in tokens]
        tokens[0] = self.seq[-1]
        M = len(tokens)
        p_draft = np.asarray(p_draft, dtype=np.float32)
        cp = self.kv_p.ctx_len[0]
        pr = self._pass_sample("p", tokens, range(cp, cp + M), p_draft, u_accept_p, u_sample_p, lam, self.criterion,
                               1, temperature, resample)
        rec = {"proxy": pr, "escalate": pr["escalate"], "catch_up": 0}
        path = pr["path"]
        if not pr["escalate"]:                                               # Case I
            self.kv_p.commit([path])
            self.seq += [tokens[i] for i in path[1:]] + [pr["token"]]
            return rec
        tau_m = pr["accepted_len"]                                           # Case II
        t_len = self.kv_t.ctx_len[0]
        unseen = self.seq[t_len:-1]
        if len(unseen) + M > self.max_nodes:
            before = self.kv_t.ctx_len[0]
            self._ingest("t", unseen)
            rec["catch_up"] = (self.kv_t.ctx_len[0] - before + self.max_nodes - 1) // self.max_nodes
            t_len, unseen = self.kv_t.ctx_len[0], []
        u = len(unseen)
        tok_t = unseen + tokens
        pd_t = np.zeros((u + M - 1, p_draft.shape[1]), dtype=np.float32)
        pd_t[u:] = p_draft                                                   # row u + i judges draft i + 1
        ua_t = np.zeros(u + M, dtype=np.float32)
        ua_t[u:] = np.asarray(u_accept_t, dtype=np.float32)
        n_forced = u + tau_m + 1
        tr = self._pass_sample("t", tok_t, range(t_len, t_len + u + M), pd_t, ua_t, u_sample_t, 0.0, CRIT_MARGIN,
                               n_forced, temperature, resample)
        self.target_passes += 1
        self.kv_t.commit([list(range(n_forced - 1)) + tr["path"]])
        extra = [n - u for n in tr["path"][1:]]                              # drafts the target accepted, chain ids
        self.kv_p.commit([path + extra])
        self.seq += [tokens[i] for i in path[1:] + extra] + [tr["token"]]
        rec.update({"target": tr, "target_nodes": u + M, "n_forced_t": n_forced})
        return rec
