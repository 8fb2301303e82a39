"""The ternary scheme's rounds (Alg. 1 of the paper) for one sequence (batch 1).

The greedy form on draft trees runs inside the library (`trispec_ternary_*`: proxy pass, routing
into Case I / Case II, prune and re-root, target pass, cache commits and target catch-up); this
class allocates the device buffers and marshals arguments.  The sampling form on draft chains
(`round_sample`) is host control flow here on top of trispec_verify / trispec_sample_decide /
trispec_kv_commit: a few dozen integers per round.
"""
from __future__ import annotations

import ctypes as C
from typing import Dict, List, Sequence

import numpy as np
import torch

from .binding import (CRIT_MARGIN, MAX_NODES, RESAMPLE_RESIDUAL, TERNARY_SCRATCH_INTS, KVCache, Model, RoundInfo,
                      SampleDecider, TernaryConfig, Verifier, check, lib)


def _aligned(n_bytes: int):
    t = torch.zeros(n_bytes + 256, dtype=torch.uint8, device="cuda")
    return t, t.data_ptr() + (-t.data_ptr()) % 256


def _pass_dict(r) -> Dict[str, object]:
    return {"accepted_len": int(r.accepted_len), "token": int(r.token), "escalate": int(r.escalate),
            "path": [int(r.path[i]) for i in range(r.path_len)]}


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
        cfg = TernaryConfig()
        cfg.proxy, cfg.target = proxy.handle, target.handle
        cfg.kv_proxy, cfg.kv_target = self.kv_p.handle, self.kv_t.handle
        cfg.workspace_proxy_bytes = proxy.workspace_bytes(1, max_nodes)
        cfg.workspace_target_bytes = target.workspace_bytes(1, max_nodes)
        self._ws_p, cfg.workspace_proxy = _aligned(cfg.workspace_proxy_bytes)
        self._ws_t, cfg.workspace_target = _aligned(cfg.workspace_target_bytes)
        self._scratch = torch.zeros(TERNARY_SCRATCH_INTS, dtype=torch.int32, device="cuda")
        cfg.scratch_dev = self._scratch.data_ptr()
        cfg.criterion, cfg.max_nodes = criterion, max_nodes
        cfg.stream = torch.cuda.current_stream().cuda_stream
        self.handle = C.c_void_p()
        check(lib().trispec_ternary_create(C.byref(cfg), C.byref(self.handle)))
        self._stale = False             # the library's copy of the sequence is behind self.seq

    def close(self):
        if self.handle:
            lib().trispec_ternary_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _pull(self, n_new: int = -1) -> None:
        """Sequence (its last n_new tokens; all of it if negative) and cache lengths as the library
        holds them now."""
        p, n = C.POINTER(C.c_int32)(), C.c_int32()
        check(lib().trispec_ternary_sequence(self.handle, C.byref(p), C.byref(n)))
        if n_new < 0 or len(self.seq) + n_new != n.value:
            self.seq = p[:n.value]
        else:
            self.seq += p[n.value - n_new:n.value]
        self.kv_p.sync_len()
        self.kv_t.sync_len()

    # -- API -------------------------------------------------------------------------------
    def start(self, prompt: Sequence[int]) -> None:
        """Caches of both models over the prompt but its last token (the first root)."""
        arr = (C.c_int32 * len(prompt))(*[int(t) for t in prompt])
        torch.cuda.current_stream().synchronize()
        check(lib().trispec_ternary_start(self.handle, arr, len(prompt)))
        self._pull()
        self._stale = False

    def resume(self, seq: Sequence[int]) -> None:
        """Take over a sequence whose caches were advanced by other means (trispec_ternary_resume)."""
        self.seq = [int(t) for t in seq]
        self.kv_p.sync_len()
        self.kv_t.sync_len()
        arr = (C.c_int32 * len(self.seq))(*self.seq)
        check(lib().trispec_ternary_resume(self.handle, arr, len(self.seq)))
        self._stale = False

    def round(self, parents: Sequence[int], tokens: Sequence[int], lam: float) -> Dict[str, object]:
        """One round on a draft tree (tokens[0] is replaced by the current root).  Returns what
        happened; self.seq has grown by the accepted drafts and one verifier token."""
        n = len(tokens)
        if self._stale:
            arr = (C.c_int32 * len(self.seq))(*self.seq)
            check(lib().trispec_ternary_resume(self.handle, arr, len(self.seq)))
            self._stale = False
        par = (C.c_int32 * n)(*[int(p) for p in parents])
        tok = (C.c_int32 * n)(*[int(t) for t in tokens])
        info = RoundInfo()
        check(lib().trispec_ternary_round(self.handle, par, tok, n, float(lam), C.byref(info)))
        self._pull(int(info.n_emitted))
        rec = {"proxy": _pass_dict(info.proxy), "escalate": int(info.escalate), "catch_up": int(info.catch_up)}
        if info.escalate:
            self.target_passes += 1
            rec.update({"target": _pass_dict(info.target), "target_nodes": int(info.target_nodes),
                        "n_forced_t": int(info.n_forced_target)})
        return rec

    # -- passes driven from here (sampling form) ------------------------------------------------
    def _pass(self, which: str, tokens, parents, positions, lam: float, criterion: int, n_forced: int):
        model, kv = (self.proxy, self.kv_p) if which == "p" else (self.target, self.kv_t)
        n = len(tokens)
        ver = self._ver.get((which, n))
        if ver is None:
            ver = self._ver[(which, n)] = Verifier(model, 1, n)
        tok = torch.tensor([list(map(int, tokens))], dtype=torch.int32, device="cuda")
        pos = torch.tensor([list(map(int, positions))], dtype=torch.int32, device="cuda")
        par = np.asarray([list(map(int, parents))], dtype=np.int32)
        ver.verify(kv, tok, par, pos, lam, criterion, n_forced, want_logits=False)
        torch.cuda.synchronize()

    def _ingest(self, which: str, tokens: Sequence[int]) -> None:
        """Plain passes over certain tokens: a forced chain, everything committed."""
        kv = self.kv_p if which == "p" else self.kv_t
        tokens = list(tokens)
        while tokens:
            chunk, tokens = tokens[: self.max_nodes], tokens[self.max_nodes:]
            n, c = len(chunk), kv.ctx_len[0]
            self._pass(which, chunk, range(-1, n - 1), range(c, c + n), 0.0, CRIT_MARGIN, n)
            kv.commit([list(range(n))])

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
            self._stale = True
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
        self._stale = True
        rec.update({"target": tr, "target_nodes": u + M, "n_forced_t": n_forced})
        return rec
