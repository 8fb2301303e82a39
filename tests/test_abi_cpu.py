"""CPU-only checks of the C ABI: the library loads, exports every symbol the header declares,
and the host-side validation returns the documented error codes without touching a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2601_23180_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    src = open(os.path.join(ROOT, "include", "trispec.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(trispec_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    syms = header_symbols()
    assert len(syms) >= 11
    for s in syms:
        assert hasattr(lib, s), s
    assert sorted(B.EXPORTS) == syms


def _cfg(**kw):
    base = dict(n_layers=2, hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=64, ffn=512, vocab=4096,
                dtype=B.TRISPEC_F32, rms_eps=1e-6, rope_base=1e4, qk_norm=0)
    base.update(kw)
    return B.ModelConfig(*[base[k] for k, _ in B.ModelConfig._fields_])


def _fake_weights(n_layers):
    w = B.Weights()
    fake = 0x1000
    w.embed = w.lm_head = w.final_norm = fake
    keep = []
    for n in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "norm_attn", "norm_ffn", "q_norm", "k_norm"):
        arr = (C.c_void_p * n_layers)(*([fake] * n_layers))
        keep.append(arr)
        setattr(w, n, C.cast(arr, C.POINTER(C.c_void_p)))
    return w, keep


def _model(**kw):
    cfg = _cfg(**kw)
    w, keep = _fake_weights(cfg.n_layers)
    h = C.c_void_p()
    rc = B.lib().trispec_model_create(C.byref(cfg), C.byref(w), C.byref(h))
    return rc, h, keep


def test_model_create_validation():
    lib = B.lib()
    assert lib.trispec_model_create(None, None, None) == -1
    assert _model()[0] == 0
    assert _model(head_dim=96)[0] == -2
    assert _model(n_q_heads=5)[0] == -2
    assert _model(dtype=7)[0] == -2
    assert _model(dtype=B.TRISPEC_BF16, hidden=250)[0] == -2
    assert _model(qk_norm=1)[0] == 0 and _model(qk_norm=2)[0] == -2
    cfg = _cfg(qk_norm=1)                      # the per-head norm weights are required when it is on
    w, keep = _fake_weights(2)
    w.q_norm = None
    h = C.c_void_p()
    assert lib.trispec_model_create(C.byref(cfg), C.byref(w), C.byref(h)) == -1
    cfg = _cfg()
    w, keep = _fake_weights(2)
    w.lm_head = None
    h = C.c_void_p()
    assert lib.trispec_model_create(C.byref(cfg), C.byref(w), C.byref(h)) == -1
    assert b"NULL" in lib.trispec_strerror(-1)


def test_kv_and_workspace_sizes():
    lib = B.lib()
    rc, m, keep = _model()
    n = C.c_size_t()
    assert lib.trispec_kv_bytes(m, 1, 256, C.byref(n)) == 0
    assert n.value == 2 * 1 * 2 * 256 * 64 * 4
    assert lib.trispec_kv_bytes(m, 1, 100, C.byref(n)) == -6      # capacity not a multiple of 64
    assert lib.trispec_kv_bytes(m, 9, 256, C.byref(n)) == -3
    assert lib.trispec_workspace_bytes(m, 1, 9, C.byref(n)) == 0 and n.value > 0
    small = n.value
    assert lib.trispec_workspace_bytes(m, 4, 60, C.byref(n)) == 0 and n.value > small
    assert lib.trispec_workspace_bytes(m, 1, 129, C.byref(n)) == -3
    assert lib.trispec_workspace_bytes(m, 8, 64, C.byref(n)) == -3  # 512 rows
    d = C.c_double()
    ctx = (C.c_int32 * 1)(128)
    assert lib.trispec_pass_bytes(m, 1, 9, ctx, C.byref(d)) == 0
    per_layer = 2 * 256 * 256 + 2 * 256 * 128 + 3 * 256 * 512 + 2 * 256
    assert d.value == (2 * per_layer + 4096 * 256 + 2 * 2 * (128 + 9) * 128) * 4
    lib.trispec_model_destroy(m)


def _verify_rc(m, kv, parents, n_nodes, *, threshold=0.5, criterion=0, n_forced=1, ws=0x10000,
               ws_bytes=1 << 40, tokens=0x2000, positions=0x3000):
    o = B.VerifyOpts(criterion, n_forced, ws, ws_bytes, None, None, None)
    out = B.VerifyOut()
    par = np.asarray(parents, dtype=np.int32)
    return B.lib().trispec_verify(m, kv, tokens, par.ctypes.data_as(C.POINTER(C.c_int32)), positions,
                                  n_nodes, threshold, C.byref(o), C.byref(out))


def test_verify_rejects_bad_arguments_before_any_launch():
    lib = B.lib()
    rc, m, keep = _model()
    kv = C.c_void_p()
    assert lib.trispec_kv_create(m, 0x4000, 0x8000, 1, 256, C.byref(kv)) == 0
    assert lib.trispec_kv_set_len(kv, (C.c_int32 * 1)(300)) == -6
    assert lib.trispec_kv_set_len(kv, (C.c_int32 * 1)(250)) == 0
    chain = [-1, 0, 1, 2]
    assert _verify_rc(m, kv, chain, 4, tokens=None) == -1
    assert _verify_rc(m, kv, chain, 0) == -3
    assert _verify_rc(m, kv, list(range(-1, 128)), 129) == -3
    assert _verify_rc(m, kv, [0, 0, 1, 2], 4) == -4            # parents[0] must be -1
    assert _verify_rc(m, kv, [-1, 0, 2, 1], 4) == -4           # parents[i] < i
    assert _verify_rc(m, kv, [-1, 0, -1, 1], 4) == -4
    assert _verify_rc(m, kv, chain, 4, n_forced=0) == -5
    assert _verify_rc(m, kv, chain, 4, n_forced=5) == -5
    assert _verify_rc(m, kv, [-1, 0, 0, 1], 4, n_forced=3) == -5   # forced nodes must be a chain
    assert _verify_rc(m, kv, chain, 4, criterion=3) == -8
    assert _verify_rc(m, kv, chain, 4, threshold=float("nan")) == -8
    assert _verify_rc(m, kv, chain, 4, ws=None) == -7
    assert _verify_rc(m, kv, chain, 4, ws=0x10010) == -7           # misaligned
    assert _verify_rc(m, kv, chain, 4, ws_bytes=1024) == -7
    assert _verify_rc(m, kv, list(range(-1, 6)), 7) == -6          # 250 + 7 > 256
    rc2, m2, keep2 = _model()
    assert _verify_rc(m2, kv, chain, 4) == -9                      # cache of another model
    lib.trispec_kv_destroy(kv)
    lib.trispec_model_destroy(m)
    lib.trispec_model_destroy(m2)


def test_copy_probe_rejects_bad_arguments_before_any_launch():
    lib = B.lib()
    assert lib.trispec_copy_probe(None, 0x1000, 1024, None) == lib.trispec_copy_probe(0x1000, None, 1024, None) < 0
    bad_size = lib.trispec_copy_probe(0x1000, 0x2000, 1000, None)       # not a multiple of 16
    bad_align = lib.trispec_copy_probe(0x1008, 0x2000, 1024, None)      # misaligned pointer
    zero = lib.trispec_copy_probe(0x1000, 0x2000, 0, None)
    assert bad_size == bad_align == zero < 0
    assert b"argument" in lib.trispec_strerror(bad_size)


def test_kv_commit_rejects_bad_arguments_before_any_launch():
    lib = B.lib()
    rc, m, keep = _model()
    kv = C.c_void_p()
    assert lib.trispec_kv_create(m, 0x4000, 0x8000, 1, 256, C.byref(kv)) == 0
    assert lib.trispec_kv_set_len(kv, (C.c_int32 * 1)(250)) == 0

    def commit(nodes, n):
        arr = (C.c_int32 * B.PATH_STRIDE)(*nodes)
        return lib.trispec_kv_commit(kv, arr, (C.c_int32 * 1)(n), None)

    assert lib.trispec_kv_commit(kv, None, (C.c_int32 * 1)(0), None) == -1
    assert commit([0, 1], 129) == -3                    # count out of range
    assert commit([0, 1], -1) == -3
    assert commit([0, 2, 2], 3) == -4                   # not strictly increasing
    assert commit([1, 0], 2) == -4
    assert commit([0, 128], 2) == -4                    # node id out of range
    assert commit([0, 3, 6], 3) == -6                   # 250 + 6 >= 256
    assert commit([], 0) == 0                           # nothing to move: no launch, length unchanged
    assert _verify_rc(m, kv, list(range(-1, 6)), 7) == -6   # still 250 cached: 250 + 7 > 256
    lib.trispec_kv_destroy(kv)
    lib.trispec_model_destroy(m)


def test_sample_decide_rejects_bad_arguments_before_any_launch():
    lib = B.lib()
    n = C.c_size_t()
    assert lib.trispec_sample_scratch_bytes(2, 9, 100, None) == -1
    assert lib.trispec_sample_scratch_bytes(0, 9, 100, C.byref(n)) == -3
    assert lib.trispec_sample_scratch_bytes(2, 65, 100, C.byref(n)) == -3
    assert lib.trispec_sample_scratch_bytes(8, 64, 100, C.byref(n)) == -3       # 512 rows
    assert lib.trispec_sample_scratch_bytes(2, 9, 0, C.byref(n)) == -8
    assert lib.trispec_sample_scratch_bytes(2, 9, 100000, C.byref(n)) == 0 and n.value >= 18 * 28 + 2 * 2 * 25 * 8
    assert lib.trispec_sample_scratch_bytes(2, 9, 100, C.byref(n)) == 0 and n.value >= 18 * 28 and n.value % 256 == 0
    out = B.VerifyOut()

    def rc(logits=0x1000, tokens=0x2000, batch=2, n_nodes=9, vocab=100, lam=0.1, T=1.0, resample=0, crit=0,
           n_forced=1, p_draft=0x3000, ua=0x4000, us=0x5000, scratch=0x10000, scratch_bytes=None):
        o = B.SampleOpts(T, resample, crit, n_forced, p_draft, ua, us, scratch,
                         n.value if scratch_bytes is None else scratch_bytes, None)
        return lib.trispec_sample_decide(logits, tokens, batch, n_nodes, vocab, lam, C.byref(o), C.byref(out))

    assert rc(logits=None) == -1 and rc(tokens=None) == -1 and rc(ua=None) == -1 and rc(us=None) == -1
    assert rc(p_draft=None) == -1
    assert rc(batch=9) == -3 and rc(n_nodes=0) == -3
    assert rc(n_forced=0) == -5 and rc(n_forced=10) == -5
    assert rc(T=0.0) == -8 and rc(T=-1.0) == -8 and rc(T=float("inf")) == -8 and rc(T=float("nan")) == -8
    assert rc(lam=float("nan")) == -8 and rc(vocab=0) == -8 and rc(resample=2) == -8 and rc(crit=5) == -8
    assert rc(scratch=None) == -7 and rc(scratch=0x10010) == -7 and rc(scratch_bytes=64) == -7


# ------------------------------------------------------------------ Case II hand-over (host integers only)

def _root_paths(parents):
    """Every root path [0, ..., v] of a tree."""
    out = []
    for v in range(len(parents)):
        p = [v]
        while parents[p[-1]] >= 0:
            p.append(int(parents[p[-1]]))
        out.append(p[::-1])
    return out


def test_prune_reroot_equals_the_oracle_on_every_root_path():
    from oracle import prune_reroot as oracle_prune
    from workloads import gen_draft_tokens, gen_eagle2_tree, gen_tree, tree_depths
    n_paths = 0
    for seed in range(6):
        for parents in (gen_tree(60, 8, 4, seed), gen_tree(23, 5, 3, seed), gen_eagle2_tree(seed), gen_tree(64, 12, 3, seed),
                        np.arange(-1, 8, dtype=np.int32), np.array([-1], dtype=np.int32)):
            tokens = gen_draft_tokens(parents, 50000, seed)
            positions = 1000 + tree_depths(parents)
            for path in _root_paths(parents):
                want = oracle_prune(tokens, parents, positions, path)
                got = B.prune_reroot(tokens, parents, positions, path)
                assert got["tokens"] == want["tokens"].tolist() and got["parents"] == want["parents"].tolist()
                assert got["positions"] == want["positions"].tolist() and got["old_id"] == want["old_id"].tolist()
                assert got["n_forced"] == want["n_forced"]
                n_paths += 1
    assert n_paths > 1000


def test_prune_reroot_with_a_prefix_equals_the_oracle_on_the_extended_tree():
    """Tokens the target has not cached ride in front: the same as pruning a tree that has them as a
    chain above its root, along the path that runs through that chain."""
    from oracle import prune_reroot as oracle_prune
    from workloads import gen_draft_tokens, gen_tree, tree_depths
    for seed, u in ((1, 1), (2, 5), (3, 17)):
        parents = gen_tree(40, 8, 4, seed)
        tokens = gen_draft_tokens(parents, 3000, seed)
        positions = 500 + u + tree_depths(parents)
        prefix = list(range(7000, 7000 + u))
        ext_par = np.concatenate([np.arange(-1, u - 1), np.where(parents < 0, u - 1, parents + u)]).astype(np.int32)
        ext_tok = np.concatenate([prefix, tokens]).astype(np.int32)
        ext_pos = np.concatenate([500 + np.arange(u), positions]).astype(np.int32)
        for path in _root_paths(parents)[::3]:
            want = oracle_prune(ext_tok, ext_par, ext_pos, list(range(u)) + [v + u for v in path])
            got = B.prune_reroot(tokens, parents, positions, path, prefix, 500)
            assert got["tokens"] == want["tokens"].tolist() and got["parents"] == want["parents"].tolist()
            assert got["positions"] == want["positions"].tolist() and got["n_forced"] == want["n_forced"]
            assert got["old_id"] == [-1] * u + [int(v) - u for v in want["old_id"][u:]]


def test_prune_reroot_errors():
    par = [-1, 0, 0, 1]
    tok, pos = [5, 6, 7, 8], [10, 11, 11, 12]
    for path, code in (([1], -4), ([0, 3], -4), ([0, 2, 3], -4), ([0, 1, 3, 3, 3], -3)):
        with pytest.raises(B.TriSpecError) as e:
            B.prune_reroot(tok, par, pos, path)
        assert e.value.code == code, (path, e.value.code)
    with pytest.raises(B.TriSpecError) as e:      # parents not topological
        B.prune_reroot(tok, [-1, 2, 0, 1], pos, [0])
    assert e.value.code == -4
    with pytest.raises(B.TriSpecError) as e:      # prefix + kept nodes exceed the node limit
        B.prune_reroot(tok, par, pos, [0], list(range(126)), 0)
    assert e.value.code == -3
    assert len(B.prune_reroot(tok, par, pos, [0], list(range(124)), 0)["tokens"]) == 128


def test_ternary_driver_rejects_bad_arguments_and_kv_len_round_trip():
    """trispec_ternary_* (Alg. 1's routing behind the boundary): what can be refused on the host is
    refused there; nothing here reaches a GPU."""
    lib = B.lib()
    _, mp, keep_p = _model()
    _, mt, keep_t = _model(n_layers=3)
    _, mv, keep_v = _model(vocab=4097)
    kvs = []
    for m, batch in ((mp, 1), (mt, 1), (mt, 2), (mv, 1)):
        h = C.c_void_p()
        assert lib.trispec_kv_create(m, 0x10000, 0x20000, batch, 256, C.byref(h)) == 0
        kvs.append(h)
    kv_p, kv_t, kv_t2, kv_v = kvs
    lens = (C.c_int32 * 2)(7, 9)
    assert lib.trispec_kv_set_len(kv_t2, lens) == 0
    got = (C.c_int32 * 2)()
    assert lib.trispec_kv_get_len(kv_t2, got) == 0 and list(got) == [7, 9]
    assert lib.trispec_kv_get_len(None, got) == -1

    def make(**kw):
        cfg = B.TernaryConfig()
        cfg.proxy, cfg.target, cfg.kv_proxy, cfg.kv_target = mp, mt, kv_p, kv_t
        cfg.workspace_proxy, cfg.workspace_target = 0x100000, 0x200000
        cfg.workspace_proxy_bytes = cfg.workspace_target_bytes = 1 << 40
        cfg.scratch_dev, cfg.criterion, cfg.max_nodes = 0x300000, B.CRIT_MARGIN, 16
        for k, v in kw.items():
            setattr(cfg, k, v)
        h = C.c_void_p()
        return lib.trispec_ternary_create(C.byref(cfg), C.byref(h)), h

    rc, t = make()
    assert rc == 0
    assert make(scratch_dev=None)[0] == -1 and make(proxy=None)[0] == -1
    assert make(max_nodes=0)[0] == -3 and make(max_nodes=129)[0] == -3
    assert make(kv_target=kv_t2)[0] == -3                        # a cache of two sequences
    assert make(kv_target=kv_p)[0] == -9                         # the other model's cache
    assert make(target=mv, kv_target=kv_v)[0] == -9              # vocabularies differ
    assert make(criterion=5)[0] == -8
    assert make(workspace_proxy_bytes=1024)[0] == -7 and make(workspace_target=None)[0] == -7
    assert lib.trispec_ternary_create(None, None) == -1
    # no sequence yet; bad trees and tokens
    par = (C.c_int32 * 4)(-1, 0, 1, 1)
    tok = (C.c_int32 * 4)(0, 5, 6, 7)
    info = B.RoundInfo()
    assert lib.trispec_ternary_round(t, par, tok, 4, 0.5, C.byref(info)) == -11
    assert lib.trispec_ternary_start(t, None, 3) == -1
    assert lib.trispec_ternary_start(t, tok, 0) == -8
    assert lib.trispec_ternary_start(t, (C.c_int32 * 2)(3, 4096), 2) == -8       # token id outside the vocabulary
    # take over a sequence of one token with empty caches (no pass needed), then argument checks of a round
    zero = (C.c_int32 * 1)(0)
    assert lib.trispec_kv_set_len(kv_p, zero) == 0 and lib.trispec_kv_set_len(kv_t, zero) == 0
    assert lib.trispec_ternary_resume(t, (C.c_int32 * 2)(3, 4), 2) == -8          # the proxy cache holds 0 tokens, not 1
    assert lib.trispec_ternary_resume(t, (C.c_int32 * 1)(3), 1) == 0
    p, n = C.POINTER(C.c_int32)(), C.c_int32()
    assert lib.trispec_ternary_sequence(t, C.byref(p), C.byref(n)) == 0 and n.value == 1 and p[0] == 3
    assert lib.trispec_ternary_round(t, par, tok, 17, 0.5, C.byref(info)) == -3   # more than max_nodes
    assert lib.trispec_ternary_round(t, (C.c_int32 * 4)(-1, 0, 2, 1), tok, 4, 0.5, C.byref(info)) == -4
    assert lib.trispec_ternary_round(t, (C.c_int32 * 4)(0, 0, 1, 1), tok, 4, 0.5, C.byref(info)) == -4
    assert lib.trispec_ternary_round(t, par, (C.c_int32 * 4)(0, 5, -1, 7), 4, 0.5, C.byref(info)) == -8
    assert lib.trispec_ternary_round(t, None, tok, 4, 0.5, C.byref(info)) == -1
    # the sampling form's round: required buffers, chain length, token ids
    ua = (C.c_float * 4)(0.1, 0.2, 0.3, 0.4)
    sr = B.SampleRound()
    sr.temperature, sr.resample = 1.0, 0
    sr.p_draft_dev, sr.logits_dev, sr.p_draft_work_dev = 0x400000, 0x500000, 0x600000
    sr.u_accept_proxy_host, sr.u_accept_target_host = ua, ua
    assert lib.trispec_ternary_round_sample(t, tok, 4, 0.5, None, C.byref(info)) == -1
    assert lib.trispec_ternary_round_sample(t, tok, 17, 0.5, C.byref(sr), C.byref(info)) == -3
    assert lib.trispec_ternary_round_sample(t, (C.c_int32 * 4)(0, 5, 4096, 7), 4, 0.5, C.byref(sr), C.byref(info)) == -8
    sr.logits_dev = None
    assert lib.trispec_ternary_round_sample(t, tok, 4, 0.5, C.byref(sr), C.byref(info)) == -1
    sr.logits_dev, sr.p_draft_dev = 0x500000, None
    assert lib.trispec_ternary_round_sample(t, tok, 4, 0.5, C.byref(sr), C.byref(info)) == -1
    assert lib.trispec_ternary_destroy(t) == 0
    for h in kvs:
        lib.trispec_kv_destroy(h)
    for m in (mp, mt, mv):
        lib.trispec_model_destroy(m)


def test_paged_cache_creation_is_validated():
    lib = B.lib()
    _, m, keep = _model()
    n = C.c_size_t()
    assert lib.trispec_kv_paged_bytes(m, 10, C.byref(n)) == 0
    assert n.value == 2 * 10 * 2 * 256 * 64 * 4                 # layers x pages x kv heads x page x head_dim x fp32
    assert lib.trispec_kv_paged_bytes(m, 0, C.byref(n)) == -6 and lib.trispec_kv_paged_bytes(m, 10, None) == -1
    h = C.c_void_p()
    ok = lambda **kw: lib.trispec_kv_create_paged(m, kw.get("k", 0x10000), kw.get("v", 0x20000), kw.get("t", 0x30000),
                                                  kw.get("batch", 2), kw.get("mp", 4), kw.get("np", 10), C.byref(h))
    assert ok() == 0
    lens = (C.c_int32 * 2)(1024, 3)
    assert lib.trispec_kv_set_len(h, lens) == 0                 # capacity = 4 pages of 256 slots
    lens[0] = 1025
    assert lib.trispec_kv_set_len(h, lens) == -6
    lib.trispec_kv_destroy(h)
    assert ok(t=None) == -1 and ok(k=None) == -1
    assert ok(batch=9) == -3 and ok(mp=0) == -6 and ok(np=0) == -6
    assert ok(k=0x10004) == -8
    lib.trispec_model_destroy(m)
