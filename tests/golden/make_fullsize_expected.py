#!/usr/bin/env python3
"""Writes tests/golden/fullsize_<case>.json: what the ORACLE computes for the full-size workloads
(workloads 2-5 of bench.py), so that the GPU parity tests at those sizes need no minutes-long CPU run.

Calls only `oracle/` and the seeded generators in `workloads/`; nothing here touches the GPU path.
The paper prints no worked numbers for a verification pass, so these are oracle values, not paper
values.  Run (about 40 minutes on 8 cores, one case at a time to bound memory):

    python tests/golden/make_fullsize_expected.py [case ...]

Each file holds the inputs that are not a pure function of the seed (planted draft tokens,
pruned trees) and, per node: argmax, confidence, margin, the two largest logits, and the logits
at a fixed sample of vocabulary indices; plus sampled entries of the K/V rows the pass appends.
Beside it, fullsize_<case>_tilecols.npz holds, per pass, the logits of every node at one column
of every 128-column vocabulary tile and at every column of the last (ragged) tile — the unit the
fused LM-head kernel works in — as float32.

    python tests/golden/make_fullsize_expected.py --tilecols-only [case ...]

recomputes only the final pass of each case from the tokens and trees the JSON file already
holds, checks that it reproduces the stored statistics, and writes just the .npz (about an hour
for all four cases on 8 cores).
"""
from __future__ import annotations

import json
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.join(HERE, "..", ".."))

from oracle import (CRIT_MARGIN, CRIT_TOP1, OracleWeights, decide, node_stats, prune_reroot,  # noqa: E402
                    verify_forward)
from workloads import (SHAPES, WeightSource, gen_chain, gen_draft_tokens, gen_kv_cache, gen_tree,  # noqa: E402
                       tree_depths)

N_SAMPLE_LOGITS = 24
N_SAMPLE_KV = 96
TILE = 128   # vocabulary columns per tile of the fused LM-head kernel


def tile_columns(vocab):
    """One column of every full 128-column tile (its place inside the tile varies from tile to
    tile) and every column of the last tile."""
    n_tiles = (vocab + TILE - 1) // TILE
    cols = [t * TILE + (t * 37 + 11) % TILE for t in range(n_tiles - 1)]
    cols += list(range((n_tiles - 1) * TILE, vocab))
    return np.asarray(cols, dtype=np.int64)


TILECOLS = {}   # pass name -> float32 [M, n_cols], filled by summarise()


def path_to(parents, node):
    p = [int(node)]
    while parents[p[-1]] >= 0:
        p.append(int(parents[p[-1]]))
    return p[::-1]


def oracle_pass(shape, seed, kv_seed, b, batch, ctx, tokens, parents, positions):
    """One sequence of a batch: synthetic cache (sequence b of the batch-wide generator)."""
    W = OracleWeights(WeightSource(shape, seed).get)
    memo = {}

    def layer_kv(l):   # K and V of a layer are generated together; keep only the current layer
        if l not in memo:
            memo.clear()
            k, v = gen_kv_cache(shape, batch, ctx, kv_seed, l)
            memo[l] = (k[b], v[b])
        return memo[l]

    return verify_forward(W, shape, lambda l: layer_kv(l)[0], lambda l: layer_kv(l)[1], tokens, parents,
                          positions)


def summarise(shape, seed, out, tokens, name):
    lg = out["logits"]
    st = node_stats(lg)
    M, V = lg.shape
    TILECOLS[name] = lg[:, tile_columns(V)].astype(np.float32)
    rng = np.random.Generator(np.random.Philox(key=[seed, 777]))
    cols = np.sort(rng.choice(V, size=N_SAMPLE_LOGITS, replace=False))
    L, nkv, _, d = out["k_new"].shape
    kv_idx = np.stack([rng.integers(0, L, N_SAMPLE_KV), rng.integers(0, nkv, N_SAMPLE_KV),
                       rng.integers(0, M, N_SAMPLE_KV), rng.integers(0, d, N_SAMPLE_KV)], axis=1)
    return {
        "tokens": [int(t) for t in tokens],
        "argmax": [int(v) for v in st["argmax"]],
        "conf": [float(v) for v in st["conf"]],
        "margin": [float(v) for v in st["margin"]],
        "l1": [float(v) for v in st["l1"]],
        "l2": [float(v) for v in st["l2"]],
        "logit_cols": [int(c) for c in cols],
        "logits": [[float(v) for v in lg[i, cols]] for i in range(M)],
        "max_abs_logit": [float(np.max(np.abs(lg[i]))) for i in range(M)],
        "kv_idx": kv_idx.tolist(),
        "k_new": [float(out["k_new"][l, h, m, j]) for l, h, m, j in kv_idx],
        "v_new": [float(out["v_new"][l, h, m, j]) for l, h, m, j in kv_idx],
    }


def planted(shape, seed, kv_seed, ctx, parents, tokens, positions, n_plant, log):
    """Plant the oracle's own greedy tokens along the path to the deepest leaf, n_plant steps."""
    tokens = tokens.copy()
    depth = tree_depths(parents)
    path = path_to(parents, int(np.argmax(depth)))
    out = None
    for step in range(n_plant + 1):
        t0 = time.time()
        out = oracle_pass(shape, seed, kv_seed, 0, 1, ctx, tokens, parents, positions)
        log(f"  pass {step} ({time.time() - t0:.0f}s)")
        if step == n_plant:
            break
        a, c = path[step], path[step + 1]
        tokens[c] = int(node_stats(out["logits"])["argmax"][a])
    return tokens, out


def case_cfg2(log):
    shape, seed, ctx = SHAPES["qwen3_0p6b"], 1002, 2048
    parents = gen_chain(9)
    tokens = gen_draft_tokens(parents, shape.vocab, seed)
    positions = (ctx + tree_depths(parents)).astype(np.int32)
    tokens, out = planted(shape, seed, seed, ctx, parents, tokens, positions, 5, log)
    return {"shape": "qwen3_0p6b", "seed": seed, "ctx": ctx, "parents": parents.tolist(),
            "positions": positions.tolist(), "seqs": [summarise(shape, seed, out, tokens, "seq0")]}


def case_cfg3(log):
    shape, seed, ctx = SHAPES["qwen3_8b"], 1003, 4096
    parents = gen_tree(60, 8, 4, seed)
    tokens = gen_draft_tokens(parents, shape.vocab, seed)
    positions = (ctx + tree_depths(parents)).astype(np.int32)
    tokens, out = planted(shape, seed, seed, ctx, parents, tokens, positions, 2, log)
    return {"shape": "qwen3_8b", "seed": seed, "ctx": ctx, "parents": parents.tolist(),
            "positions": positions.tolist(), "seqs": [summarise(shape, seed, out, tokens, "seq0")]}


def case_cfg4(log):
    """Proxy pass on the full tree; for every (criterion, threshold) of the sweep the oracle's
    decision; for every distinct escalation the pruned / re-rooted target pass (Eq. 10).
    Seed 2004 rather than 1004: with it the oracle's proxy is confident at the root (top-1
    probability 0.905), so the sweep escalates part-way down the planted path and the target pass
    sees a pruned tree with a forced chain, not only the whole tree."""
    pshape, tshape, seed, tseed, ctx = SHAPES["qwen3_1p7b"], SHAPES["qwen3_8b"], 2004, 2014, 8192
    parents = gen_tree(60, 8, 4, seed)
    tokens = gen_draft_tokens(parents, pshape.vocab, seed)
    positions = (ctx + tree_depths(parents)).astype(np.int32)
    tokens, out = planted(pshape, seed, seed, ctx, parents, tokens, positions, 3, log)
    st = node_stats(out["logits"])
    res = {"proxy_shape": "qwen3_1p7b", "target_shape": "qwen3_8b", "seed": seed, "target_seed": tseed,
           "ctx": ctx, "parents": parents.tolist(), "positions": positions.tolist(),
           "proxy": summarise(pshape, seed, out, tokens, "proxy"), "routes": [], "targets": {}}
    for crit, cname in ((CRIT_TOP1, "top1"), (CRIT_MARGIN, "margin")):
        for lam in (0.5, 0.7, 0.9):
            dec = decide(tokens, parents, st["argmax"], st["conf"], st["margin"], lam, crit, 1)
            route = {"criterion": cname, "threshold": lam, "accepted_len": int(dec["accepted_len"]),
                     "token": int(dec["token"]), "escalate": int(dec["escalate"]),
                     "path": [int(v) for v in dec["path"]]}
            if dec["escalate"]:
                key = ",".join(str(v) for v in route["path"])
                route["target"] = key
                if key not in res["targets"]:
                    pr = prune_reroot(tokens, parents, positions, dec["path"])
                    log(f"  target pass for path [{key}]: {len(pr['tokens'])} nodes, n_forced {pr['n_forced']}")
                    t0 = time.time()
                    tout = oracle_pass(tshape, tseed, tseed, 0, 1, ctx, pr["tokens"], pr["parents"], pr["positions"])
                    log(f"  done ({time.time() - t0:.0f}s)")
                    s = summarise(tshape, tseed, tout, pr["tokens"], "target:" + key)
                    ts = node_stats(tout["logits"])
                    td = decide(pr["tokens"], pr["parents"], ts["argmax"], ts["conf"], ts["margin"], 0.0,
                                CRIT_MARGIN, pr["n_forced"])
                    s.update({"parents": [int(v) for v in pr["parents"]], "positions": [int(v) for v in pr["positions"]],
                              "n_forced": int(pr["n_forced"]),
                              "decision": {"accepted_len": int(td["accepted_len"]), "token": int(td["token"]),
                                           "escalate": int(td["escalate"]), "path": [int(v) for v in td["path"]]}})
                    res["targets"][key] = s
            res["routes"].append(route)
    return res


def case_cfg5(log):
    shape, seed, ctx, batch = SHAPES["llama3_8b"], 1005, 16384, 4
    seqs, par, pos = [], [], []
    for b in range(batch):
        parents = gen_tree(60, 8, 4, seed + b)
        tokens = gen_draft_tokens(parents, shape.vocab, seed + b)
        positions = (ctx + tree_depths(parents)).astype(np.int32)
        t0 = time.time()
        out = oracle_pass(shape, seed, seed, b, batch, ctx, tokens, parents, positions)
        log(f"  sequence {b} ({time.time() - t0:.0f}s)")
        seqs.append(summarise(shape, seed + b, out, tokens, f"seq{b}"))
        par.append(parents.tolist()); pos.append(positions.tolist())
    return {"shape": "llama3_8b", "seed": seed, "ctx": ctx, "batch": batch, "parents": par, "positions": pos,
            "seqs": seqs}


CASES = {"cfg2": case_cfg2, "cfg3": case_cfg3, "cfg4": case_cfg4, "cfg5": case_cfg5}


def tilecols_only(name, log):
    """The final pass of every sequence / target of a case, from the tokens and trees its JSON
    file holds; the stored statistics must come out again."""
    with open(os.path.join(HERE, f"fullsize_{name}.json")) as f:
        g = json.load(f)

    def redo(shape, seed, kv_seed, b, batch, stored, parents, positions, key):
        t0 = time.time()
        out = oracle_pass(shape, seed, kv_seed, b, batch, g["ctx"], np.asarray(stored["tokens"], dtype=np.int32),
                          np.asarray(parents, dtype=np.int32), np.asarray(positions, dtype=np.int32))
        st = node_stats(out["logits"])
        assert [int(v) for v in st["argmax"]] == stored["argmax"], key
        assert np.allclose(st["l1"], stored["l1"], rtol=0, atol=1e-9) and np.allclose(st["conf"], stored["conf"], rtol=0, atol=1e-12), key
        TILECOLS[key] = out["logits"][:, tile_columns(shape.vocab)].astype(np.float32)
        log(f"  {key} ({time.time() - t0:.0f}s)")

    if name == "cfg4":
        redo(SHAPES[g["proxy_shape"]], g["seed"], g["seed"], 0, 1, g["proxy"], g["parents"], g["positions"], "proxy")
        for key, t in g["targets"].items():
            redo(SHAPES[g["target_shape"]], g["target_seed"], g["target_seed"], 0, 1, t, t["parents"], t["positions"],
                 "target:" + key)
    else:
        batch = g.get("batch", 1)
        for b, s in enumerate(g["seqs"]):
            par = g["parents"][b] if batch > 1 else g["parents"]
            pos = g["positions"][b] if batch > 1 else g["positions"]
            redo(SHAPES[g["shape"]], g["seed"], g["seed"], b, batch, s, par, pos, f"seq{b}")


def main():
    args = sys.argv[1:]
    only = "--tilecols-only" in args
    names = [a for a in args if not a.startswith("--")] or list(CASES)
    for name in names:
        t0 = time.time()

        def log(msg):
            print(f"[{name} +{time.time() - t0:.0f}s] {msg}", flush=True)

        log("start")
        TILECOLS.clear()
        if only:
            tilecols_only(name, log)
        else:
            res = CASES[name](log)
            path = os.path.join(HERE, f"fullsize_{name}.json")
            with open(path, "w") as f:
                json.dump(res, f, separators=(",", ":"))
                f.write("\n")
            log(f"wrote {path}")
        path = os.path.join(HERE, f"fullsize_{name}_tilecols.npz")
        np.savez_compressed(path, **TILECOLS)
        log(f"wrote {path}")


if __name__ == "__main__":
    main()
