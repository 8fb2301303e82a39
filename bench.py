#!/usr/bin/env python3
"""Benchmark of the TriSpec verification pass on one MI355X.

A step = one trispec_verify() call: the whole hot path (embedding, every layer's projections,
tree-masked attention and FFN, fused LM head, decision) over one batch of synthetic input that
is already resident in HBM.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E vendor peak

# name -> (shape key, batch, ctx_len, n_nodes, tree kind)
WORKLOADS = {
    "qwen3_8b_tree60_ctx4096": ("qwen3_8b", 1, 4096, 60, "tree"),        # workload 3 (headline)
    "qwen3_0p6b_chain8_ctx2048": ("qwen3_0p6b", 1, 2048, 9, "chain"),    # workload 2
    "qwen3_1p7b_tree60_ctx8192": ("qwen3_1p7b", 1, 8192, 60, "tree"),    # workload 4, proxy
    "qwen3_8b_tree60_ctx8192": ("qwen3_8b", 1, 8192, 60, "tree"),        # workload 4, target
    "llama3_8b_b4_tree60_ctx16384": ("llama3_8b", 4, 16384, 60, "tree"),  # workload 5
    "tiny_bf16_tree60_ctx256": ("tiny_bf16", 1, 256, 60, "tree"),        # plumbing check only
    "qwen3_8b_4layers_tree60_ctx4096": ("qwen3_8b_L4", 1, 4096, 60, "tree"),  # kernel tuning aid (not a result)
}


def build_inputs(shape, batch, ctx, n_nodes, kind, seed):
    import torch
    from paper_2601_23180_amd import KVCache, Verifier, fill_kv_layer, model_from_arrays
    from workloads import (WeightSource, gen_chain, gen_draft_tokens, gen_kv_cache, gen_tree, tree_depths)

    ws = WeightSource(shape, seed)
    t0 = time.time()
    model = model_from_arrays(shape, ws.bits if shape.dtype == "bf16" else ws.get)
    cap = (ctx + n_nodes + 63) // 64 * 64
    kv = KVCache(model, batch, cap)
    for l in range(shape.n_layers):
        k, v = gen_kv_cache(shape, batch, ctx, seed, l)
        fill_kv_layer(kv, l, k, v)
    kv.set_len([ctx] * batch)
    parents = np.stack([gen_chain(n_nodes) if kind == "chain" else gen_tree(n_nodes, 8, 4, seed + b)
                        for b in range(batch)])
    tokens = np.stack([gen_draft_tokens(parents[b], shape.vocab, seed + b) for b in range(batch)])
    positions = np.stack([ctx + tree_depths(parents[b]) for b in range(batch)]).astype(np.int32)
    ver = Verifier(model, batch, n_nodes)
    tok = torch.from_numpy(tokens).cuda()
    pos = torch.from_numpy(positions).cuda()
    torch.cuda.synchronize()
    return dict(model=model, kv=kv, ver=ver, tok=tok, pos=pos, parents=parents, tokens=tokens,
                positions=positions, setup_s=time.time() - t0)


def cpu_baseline(shape, batch, ctx, n_nodes, kind, seed):
    """The oracle as it stands, timed on the host cores on a bounded sample of the workload:
    the full-width model cut to 2 and to 10 layers (full LM head both times), sequence 0 only,
    about 10 s of oracle time; the per-layer time is the difference / 8 and the whole pass is
    extrapolated from it."""
    from oracle import OracleWeights, verify_forward
    from workloads import WeightSource, gen_chain, gen_draft_tokens, gen_kv_cache, gen_tree, tree_depths

    ws = WeightSource(shape, seed)
    cache = {}

    def get(name, layer):   # weights generated outside the timed region
        return cache[(name, layer)]

    for name in ("embed", "lm_head", "final_norm"):
        cache[(name, 0)] = ws.get(name, 0)
    cuts = (2, 10) if shape.n_layers >= 10 else (1, min(4, shape.n_layers))
    for l in range(cuts[1]):
        for name in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_ffn"):
            cache[(name, l)] = ws.get(name, l)
    kvs = [tuple(a[0] for a in gen_kv_cache(shape, 1, ctx, seed, l)) for l in range(cuts[1])]
    parents = gen_chain(n_nodes) if kind == "chain" else gen_tree(n_nodes, 8, 4, seed)
    tokens = gen_draft_tokens(parents, shape.vocab, seed)
    positions = ctx + tree_depths(parents)
    W = OracleWeights(get)
    times = []
    for nl in cuts:
        sh = shape.with_(n_layers=nl)
        t0 = time.perf_counter()
        verify_forward(W, sh, lambda l: kvs[l][0], lambda l: kvs[l][1], tokens, parents, positions)
        times.append(time.perf_counter() - t0)
    per_layer = max((times[1] - times[0]) / (cuts[1] - cuts[0]), 1e-9)
    full = (times[0] + (shape.n_layers - 1) * per_layer) * batch
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": batch * (n_nodes - 1) / full, "unit": "draft tokens/s", "cores": int(cores),
            "kind": "oracle", "seconds_per_pass_extrapolated": full,
            "sample": f"numpy fp64 oracle, sequence 0, model cut to {cuts[0]} and {cuts[1]} layers at full width + "
                      f"full LM head ({times[0]:.2f}s, {times[1]:.2f}s); per layer = (t{cuts[1]}-t{cuts[0]})/{cuts[1] - cuts[0]}, "
                      f"pass = t{cuts[0]} + (L-{cuts[0]})*per layer, times batch"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="qwen3_8b_tree60_ctx4096", choices=sorted(WORKLOADS))
    ap.add_argument("--seed", type=int, default=1003)
    ap.add_argument("--threshold", type=float, default=0.5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--launch-mode", choices=("per-matmul", "per-layer"), default="per-matmul",
                    help="per-matmul: one launch per matmul (default, the faster cut); per-layer: the matmuls "
                         "between two attention calls as one launch with device-side barriers")
    ap.add_argument("--launch", choices=("eager", "graph"), default="eager",
                    help="graph: the pass is captured once into a HIP graph and the timed steps replay it")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs the verification pass on ONE GPU (no sharding, no collectives); "
                 "use --gpus 1")

    import torch
    from paper_2601_23180_amd.binding import LIB_PATH
    if not os.path.exists(LIB_PATH):     # load what is built; build only if nothing is
        from paper_2601_23180_amd.build import build
        build()
    from paper_2601_23180_amd import K_ATTN, K_GEMM, K_HEAD, KernelTimer
    from workloads import SHAPES

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU (there is no CPU fallback of the product path)")
    key, batch, ctx, n_nodes, kind = WORKLOADS[args.workload]
    shape = SHAPES["qwen3_8b"].with_(n_layers=4) if key == "qwen3_8b_L4" else SHAPES[key]
    inp = build_inputs(shape, batch, ctx, n_nodes, kind, args.seed)
    ver, kv, tok, pos, parents = inp["ver"], inp["kv"], inp["tok"], inp["pos"], inp["parents"]
    from paper_2601_23180_amd.binding import LAUNCH_PER_LAYER, LAUNCH_PER_MATMUL
    ver.launch_mode = LAUNCH_PER_LAYER if args.launch_mode == "per-layer" else LAUNCH_PER_MATMUL

    def step():
        ver.verify(kv, tok, parents, pos, args.threshold, want_logits=False)

    timed_step = step
    if args.launch == "graph":
        # the library only launches kernels on the caller's stream (no allocation, no memset, no
        # host synchronisation), so a pass can be captured as it is
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        timed_step = graph.replay
    for _ in range(args.warmup):
        timed_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        timed_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms = dt / args.steps * 1e3
    pass_bytes = inp["model"].pass_bytes(batch, n_nodes, [ctx] * batch)

    # per-kernel durations: HIP events on the pass's stream around every launch of one class,
    # over `steps` more passes each (same inputs, same launch configuration)
    kernels = {}
    for cls, name, per_pass in ((K_GEMM, "gemm", 4 * shape.n_layers), (K_HEAD, "lm_head", 1),
                                (K_ATTN, "attention", shape.n_layers)):
        timer = KernelTimer(cls, per_pass * args.steps)
        ver.timer = timer
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        n, tms, by = timer.read()
        ver.timer = None
        kernels[name] = {"launches": n, "avg_us": tms / n * 1e3, "bytes_per_launch": by / n,
                         "achieved_GBs": by / (tms * 1e-3) / 1e9, "ms_per_pass": tms / args.steps}
    # measured streaming ceiling of this card: a plain copy of 1 GiB (read + write counted)
    from paper_2601_23180_amd import copy_probe
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    copy_probe(dst, src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        copy_probe(dst, src)
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst

    # HBM traffic of the dominant kernel from the committed counter summary of the same command
    # (two rocprofv3 --pmc runs, scaled by the copy kernel of known size; see profiles/)
    traffic, traffic_note = None, None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{args.workload}.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            tj = json.load(f)
        traffic, traffic_note = tj.get("gemm_bytes_per_launch"), tj.get("source")

    g = kernels["gemm"]
    roofline = {"bound": "hbm", "kernel": "k_gemm_bf16 (weight-streaming projection / FFN matmul)",
                "achieved": g["achieved_GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": g["achieved_GBs"] / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_note,
                "avg_launch_us": g["avg_us"], "bytes_per_launch": g["bytes_per_launch"]}

    out = {
        "metric": "draft_tokens_verified_per_sec", "value": batch * (n_nodes - 1) / (ms * 1e-3),
        "unit": "draft tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if shape.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "batch": batch, "ctx_len": ctx, "n_nodes": n_nodes,
                   "tree": kind, "threshold": args.threshold, "launch": args.launch},
        "verify_latency_ms": ms,
        "pass_bytes": pass_bytes,
        "pass_achieved_GBs": pass_bytes / (ms * 1e-3) / 1e9,
        "pass_frac_of_hbm_peak": pass_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "roofline": roofline,
        "copy_ceiling_GBs": copy_gbs,
        "kernels": kernels,
        "accepted_len": ver.out["accepted_len"].cpu().tolist(),
        "escalate": ver.out["escalate"].cpu().tolist(),
        "setup_seconds": inp["setup_s"],
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, batch, ctx, n_nodes, kind, args.seed)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
