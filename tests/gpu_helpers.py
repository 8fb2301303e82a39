"""GPU-side test helpers: build a device model + cache from the seeded generators, run the
HIP path and the oracle on the same inputs."""
import numpy as np
import torch

from oracle import (CRIT_ENTROPY, CRIT_MARGIN, OracleWeights, causal_forward, decide, node_stats, tie_flags,
                    verify_forward)
from paper_2601_23180_amd import KVCache, Model, PagedKVCache, Verifier, fill_kv_layer, model_from_arrays
from workloads import WeightSource, gen_kv_cache, tree_depths


def device_model(shape, seed):
    ws = WeightSource(shape, seed)
    get = ws.bits if shape.dtype == "bf16" else ws.get
    return model_from_arrays(shape, get)


def capacity_for(n):
    return (n + 63) // 64 * 64


class Case:
    """One verify problem: a model, per-sequence context K/V (oracle layout [L, n_kv, C, d]),
    draft tokens / parents / positions per sequence."""

    def __init__(self, shape, seed, k_ctx, v_ctx, tokens, parents, positions):
        self.shape, self.seed = shape, seed
        self.k_ctx, self.v_ctx = k_ctx, v_ctx           # lists over batch
        self.tokens = np.asarray(tokens, dtype=np.int32).reshape(len(k_ctx), -1)
        self.parents = np.asarray(parents, dtype=np.int32).reshape(len(k_ctx), -1)
        self.positions = np.asarray(positions, dtype=np.int32).reshape(len(k_ctx), -1)
        self.batch, self.n_nodes = self.tokens.shape
        self.ctx_len = [k.shape[2] for k in k_ctx]

    def run_oracle(self):
        W = OracleWeights(WeightSource(self.shape, self.seed).get)
        outs = []
        for b in range(self.batch):
            o = verify_forward(W, self.shape, self.k_ctx[b], self.v_ctx[b], self.tokens[b], self.parents[b],
                               self.positions[b])
            o["stats"] = node_stats(o["logits"])
            outs.append(o)
        return outs

    def run_gpu(self, threshold, criterion=CRIT_MARGIN, n_forced=1, model=None, want_logits=True,
                export_hidden=False, launch_mode=0, paged=False):
        model = model or device_model(self.shape, self.seed)
        cap = capacity_for(max(self.ctx_len) + self.n_nodes)
        kv = PagedKVCache(model, self.batch, cap, seed=self.seed) if paged else KVCache(model, self.batch, cap)
        cap = kv.capacity
        c = model.cfg
        dt = torch.float32 if self.shape.dtype == "f32" else torch.bfloat16
        # poison the unused slots (and, paged, the unmapped pages) so that a kernel reading them shows up
        kd = torch.full((c.n_layers, self.batch, c.n_kv_heads, cap, c.head_dim), float("nan"), dtype=dt, device="cuda")
        vd = torch.full((c.n_layers, self.batch, c.n_kv_heads, c.head_dim, cap), float("nan"), dtype=dt, device="cuda")
        if paged:
            kv.k_pool.fill_(float("nan")); kv.v_pool.fill_(float("nan"))
        for l in range(self.shape.n_layers):
            for b in range(self.batch):
                C = self.ctx_len[b]
                kt = torch.from_numpy(np.asarray(self.k_ctx[b][l], dtype=np.float32)).cuda().to(dt)
                vt = torch.from_numpy(np.asarray(self.v_ctx[b][l], dtype=np.float32)).cuda().to(dt)
                kd[l, b, :, :C, :] = kt
                vd[l, b, :, :, :C] = vt.transpose(-1, -2)
        kv.load_dense(kd, vd)
        del kd, vd
        kv.set_len(self.ctx_len)
        ver = Verifier(model, self.batch, self.n_nodes, debug_logits=want_logits, export_hidden=export_hidden)
        ver.launch_mode = launch_mode
        tok = torch.from_numpy(self.tokens).cuda()
        pos = torch.from_numpy(self.positions).cuda()
        out = ver.verify(kv, tok, self.parents, pos, threshold, criterion, n_forced)
        torch.cuda.synchronize()
        res = {k: v.cpu().numpy().copy() for k, v in out.items()}
        if want_logits:
            res["logits"] = ver.logits.cpu().numpy().copy()
        if export_hidden:
            res["hidden"] = ver.hidden.cpu().numpy().copy()
        res["_ver"], res["_kv"], res["_model"], res["_tok"] = ver, kv, model, tok
        return res


def oracle_decision(case, oracle_out, b, threshold, criterion, n_forced=1):
    st = oracle_out[b]["stats"]
    return decide(case.tokens[b], case.parents[b], st["argmax"], st["conf"], st["margin"], threshold,
                  criterion, n_forced, entropy=st["entropy"])


def tie_resolutions(case, oracle_out, b, threshold, criterion, n_forced, nodes, tol=1e-3):
    """Every decision the oracle reaches when the ties on `nodes` are resolved the other way: a
    routing statistic within tol of the threshold may fall on either side of it, and of two top
    logits within tol of each other either may be the argmax."""
    import itertools
    st = oracle_out[b]["stats"]
    stat = st["entropy"] if criterion == CRIT_ENTROPY else (st["margin"] if criterion == CRIT_MARGIN else st["conf"])
    logits = oracle_out[b]["logits"]
    options = []
    for i in nodes:
        flips = []                       # the independent flips this node allows
        if abs(stat[i] - threshold) < tol:
            flips.append(("g", i))
        if st["l1"][i] - st["l2"][i] < tol:
            flips.append(("a", i))
        # every subset of them
        options.append([tuple(f for k, f in enumerate(flips) if m >> k & 1) for m in range(1 << len(flips))])
    out = []
    for combo in itertools.islice(itertools.product(*options), 256):
        argmax, conf, margin, ent = st["argmax"].copy(), st["conf"].copy(), st["margin"].copy(), st["entropy"].copy()
        for c in combo:
            for kind, i in c:
                if kind == "g":       # the other side of the threshold
                    conf[i] = margin[i] = (threshold - 1.0) if stat[i] >= threshold else (threshold + 1.0)
                    ent[i] = (threshold + 1.0) if stat[i] <= threshold else (threshold - 1.0)
                else:                 # the runner-up as the argmax
                    order = np.argsort(-logits[i], kind="stable")
                    argmax[i] = order[1]
        out.append(decide(case.tokens[b], case.parents[b], argmax, conf, margin, threshold, criterion, n_forced,
                          entropy=ent))
    return out


def compare_decisions(case, gpu, oracle_out, threshold, criterion, n_forced=1):
    """Bit-exact accepted_len / token / escalate / path / argmax unless the oracle flags a tie
    (statistic within 1e-3 of the threshold, or top-2 logit gap below 1e-3) on a node the walk
    can reach — and then the GPU's answer must be the oracle's answer under another resolution of
    those ties; returns the number of tie-excused sequences."""
    excused = 0
    for b in range(case.batch):
        st = oracle_out[b]["stats"]
        flags = tie_flags(st, threshold, criterion)
        want = oracle_decision(case, oracle_out, b, threshold, criterion, n_forced)
        got_path = [int(v) for v in gpu["path"][b] if v >= 0]
        got = (int(gpu["accepted_len"][b]), int(gpu["token"][b]), int(gpu["escalate"][b]), got_path)
        same = got == (want["accepted_len"], want["token"], want["escalate"], list(want["path"]))
        touched = sorted(set(want["path"]) | set(got_path))
        if not same:
            tied = [i for i in touched if flags[i]]
            assert tied, (b, want, got)
            alts = tie_resolutions(case, oracle_out, b, threshold, criterion, n_forced, tied)
            assert any(got == (a["accepted_len"], a["token"], a["escalate"], list(a["path"])) for a in alts), (b, want, got)
            excused += 1
        gap_ok = (st["l1"] - st["l2"]) >= 1e-3
        assert np.array_equal(gpu["argmax"][b][gap_ok], st["argmax"][gap_ok])
    return excused
