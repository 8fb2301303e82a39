"""The ternary scheme's rounds (Alg. 1 of the paper) for one sequence (batch 1).

The rounds run inside the library (`trispec_ternary_*`: proxy pass, routing into Case I /
Case II, prune and re-root, target pass, cache commits and target catch-up); this
class allocates the device buffers and marshals arguments, for the greedy form on draft trees
(`round`) and the sampling form on draft chains (`round_sample`).
"""
from __future__ import annotations

import ctypes as C
from typing import Dict, List, Sequence

import numpy as np
import torch

from .binding import (CRIT_MARGIN, MAX_NODES, RESAMPLE_RESIDUAL, TERNARY_SCRATCH_INTS, KVCache, Model, PagedKVCache, RoundInfo,
                      SampleRound, TernaryConfig, check, lib)


def _aligned(n_bytes: int):
    t = torch.zeros(n_bytes + 256, dtype=torch.uint8, device="cuda")
    return t, t.data_ptr() + (-t.data_ptr()) % 256


def _pass_dict(r) -> Dict[str, object]:
    return {"accepted_len": int(r.accepted_len), "token": int(r.token), "escalate": int(r.escalate),
            "path": [int(r.path[i]) for i in range(r.path_len)]}


class TernaryDecoder:
    def __init__(self, proxy: Model, target: Model, capacity: int, criterion: int = CRIT_MARGIN,
                 max_nodes: int = MAX_NODES, paged: bool = False):
        self.proxy, self.target = proxy, target
        cache = PagedKVCache if paged else KVCache
        self.kv_p, self.kv_t = cache(proxy, 1, capacity), cache(target, 1, capacity)
        self.criterion, self.max_nodes = criterion, max_nodes
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
        self._logits = self._pd_work = None   # work buffers of the sampling form, made on first use

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

    def round_sample(self, tokens: Sequence[int], p_draft: np.ndarray, u_accept_p, u_sample_p: float, u_accept_t,
                     u_sample_t: float, lam: float, temperature: float,
                     resample: int = RESAMPLE_RESIDUAL) -> Dict[str, object]:
        """One round at temperature > 0 on a draft chain tokens[0..k] (tokens[0] is replaced by the
        current root): p_draft [k, vocab] are the drafter's distributions, the uniforms are the
        caller's.  The proxy accepts by Eq. 6 and routes by Eq. 8 / 9; on escalation the target
        verifies the whole chain with x_1..x_tau_m taken as approved (trispec_ternary_round_sample)."""
        n, vocab = len(tokens), self.proxy.cfg.vocab
        if self._stale:
            self.resume(self.seq)
        if self._logits is None:
            f32 = dict(dtype=torch.float32, device="cuda")
            self._logits = torch.zeros((self.max_nodes, vocab), **f32)
            self._pd_work = torch.zeros((max(self.max_nodes - 1, 1), vocab), **f32)
        pd = torch.as_tensor(np.ascontiguousarray(p_draft, dtype=np.float32), dtype=torch.float32, device="cuda")
        s = SampleRound()
        s.temperature, s.resample = float(temperature), int(resample)
        s.p_draft_dev = pd.data_ptr() if n > 1 else None
        ua_p = (C.c_float * n)(*[float(u) for u in u_accept_p])
        ua_t = (C.c_float * n)(*[float(u) for u in u_accept_t])
        s.u_accept_proxy_host, s.u_accept_target_host = ua_p, ua_t
        s.u_sample_proxy, s.u_sample_target = float(u_sample_p), float(u_sample_t)
        s.logits_dev, s.p_draft_work_dev = self._logits.data_ptr(), self._pd_work.data_ptr()
        tok = (C.c_int32 * n)(*[int(t) for t in tokens])
        info = RoundInfo()
        torch.cuda.current_stream().synchronize()          # p_draft is on the device before the library reads it
        check(lib().trispec_ternary_round_sample(self.handle, tok, n, float(lam), C.byref(s), C.byref(info)))
        self._pull(int(info.n_emitted))
        rec = {"proxy": _pass_dict(info.proxy), "escalate": int(info.escalate), "catch_up": int(info.catch_up)}
        if info.escalate:
            self.target_passes += 1
            rec.update({"target": _pass_dict(info.target), "target_nodes": int(info.target_nodes),
                        "n_forced_t": int(info.n_forced_target)})
        return rec
