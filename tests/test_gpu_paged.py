"""The paged cache layout (trispec_kv_create_paged): the same pass, decision, cache append and
commit as with the contiguous cache, through a shuffled page table with unmapped spare pages.
Every case goes against the CPU oracle with the bars of test_gpu_parity.py; what the layouts must
share exactly (appended K/V, committed rows) is compared bit for bit between the two."""
import numpy as np
import pytest
import torch

from oracle import CRIT_MARGIN
from paper_2601_23180_amd import KVCache, PagedKVCache
from workloads import SHAPES, gen_chain, gen_context_tokens, gen_draft_tokens, gen_tree, tree_depths
from gpu_helpers import Case, device_model
from helpers import oracle_weights
from test_gpu_parity import LAYER_SHAPE, TB, full_check, make_case

pytestmark = pytest.mark.gpu

PAGED_CASES = [
    # contexts of one, two and five pages; batches with ragged and empty contexts; both head sizes; fp32
    ("chain9_one_page", TB, [128], lambda s: gen_chain(9), 0),
    ("tree60_two_pages", TB, [300], lambda s: gen_tree(60, 8, 4, s), 0),
    ("tree_crossing_a_page_end", TB, [250], lambda s: gen_tree(24, 6, 3, s), 0),      # draft slots 250 .. 273
    ("five_pages_many_splits", TB.with_(n_layers=1), [1100], lambda s: gen_tree(33, 8, 4, s), 0),
    ("batch3_ragged_ctx", TB, [10, 400, 0], lambda s: gen_tree(30, 6, 4, s), 0),
    ("head_dim64_group2", TB.with_(head_dim=64, n_q_heads=8, n_kv_heads=4), [270], lambda s: gen_tree(40, 6, 4, s), 0),
    ("batch4_rows240", TB.with_(n_layers=1), [40, 0, 257, 77], lambda s: gen_tree(60, 8, 4, s), 0),
    ("per_layer_launch", LAYER_SHAPE, [280], lambda s: gen_tree(60, 8, 4, s), 1),
    ("fp32_model", SHAPES["tiny"], [300], lambda s: gen_tree(20, 6, 3, s), 0),
]


@pytest.mark.parametrize("name,shape,ctx_lens,tree,mode", PAGED_CASES, ids=[c[0] for c in PAGED_CASES])
def test_paged_cache_against_the_oracle(name, shape, ctx_lens, tree, mode):
    seed = 70 + len(name)
    parents = [tree(seed + b) for b in range(len(ctx_lens))]
    case = make_case(shape, seed, ctx_lens, parents)
    gpu, oracle_out, _ = full_check(case, thresholds=(0.0, 0.5), launch_mode=mode, paged=True)
    kv = gpu["_kv"]
    assert isinstance(kv, PagedKVCache) and kv.n_pages > kv.batch * kv.max_pages
    # pages that the table does not map were never written (still the harness's poison)
    mapped = set(kv.table.flatten().tolist())
    spare = [p for p in range(kv.n_pages) if p not in mapped]
    assert spare and torch.isnan(kv.k_pool[:, spare].float()).all() and torch.isnan(kv.v_pool[:, spare].float()).all()


def test_long_contexts_paged():
    """Contexts beyond what the oracle can prefill (N(0,1) caches): 40000 keys (157 pages, 63 key
    splits), and a two-sequence batch of 240 rows per kv head that takes the 256-row workgroups."""
    from workloads import gen_kv_cache
    for ctx_lens, n_nodes, n_q_heads in (((40000,), 33, 4), ((6500, 300), 60, 8)):
        shape, seed = TB.with_(n_layers=1, n_q_heads=n_q_heads), 33
        batch = len(ctx_lens)
        parents = [gen_tree(n_nodes, 8, 4, seed + b) for b in range(batch)]
        k, v = gen_kv_cache(shape, batch, max(ctx_lens), seed, 0)
        case = Case(shape, seed,
                    [k[b][None, :, :n].astype(np.float64) for b, n in enumerate(ctx_lens)],
                    [v[b][None, :, :n].astype(np.float64) for b, n in enumerate(ctx_lens)],
                    np.stack([gen_draft_tokens(p_, shape.vocab, seed + b) for b, p_ in enumerate(parents)]),
                    np.stack(parents), np.stack([n + tree_depths(p_) for n, p_ in zip(ctx_lens, parents)]))
        full_check(case, thresholds=(0.0, 0.5), paged=True)


def test_appended_rows_are_the_same_bits_in_both_layouts():
    """The K/V rows a pass appends depend on the layout only through where they are stored."""
    shape = TB
    case = make_case(shape, 9, [250], [gen_tree(24, 6, 3, 9)])        # slots 250 .. 273: two pages
    model = device_model(shape, case.seed)
    a = case.run_gpu(0.5, model=model)
    b = case.run_gpu(0.5, model=model, paged=True)
    C, M = 250, 24
    ka, va, kb, vb = a["_kv"].k, a["_kv"].v, b["_kv"].k, b["_kv"].v
    assert torch.equal(ka[:, :, :, C:C + M, :], kb[:, :, :, C:C + M, :])
    assert torch.equal(va[:, :, :, :, C:C + M], vb[:, :, :, :, C:C + M])
    assert torch.isnan(kb[:, :, :, C + M:, :].float()).all() and torch.isnan(vb[:, :, :, :, C + M:].float()).all()
    assert torch.equal(ka[:, :, :, :C, :], kb[:, :, :, :C, :])
    for key in ("accepted_len", "token", "escalate", "path", "argmax"):
        assert np.array_equal(a[key], b[key]), key
    assert np.abs(a["logits"] - b["logits"]).max() <= 2e-3            # key splits start elsewhere: not the same sums


def test_commit_moves_exactly_the_path_rows_between_pages():
    model = device_model(SHAPES["tiny_bf16"], 5)
    kv = PagedKVCache(model, 2, 512, seed=11)
    g = torch.Generator(device="cuda").manual_seed(1)
    kv.k_pool.copy_(torch.randn(kv.k_pool.shape, device="cuda", generator=g).to(kv.k_pool.dtype))
    kv.v_pool.copy_(torch.randn(kv.v_pool.shape, device="cuda", generator=g).to(kv.v_pool.dtype))
    k0, v0 = kv.k.clone(), kv.v.clone()
    pools = kv.k_pool.clone(), kv.v_pool.clone()
    ctx = [250, 17]                                   # the first path's rows move across a page end
    kv.set_len(ctx)
    paths = [[0, 3, 4, 11, 19], [2]]
    kv.commit(paths)
    torch.cuda.synchronize()
    assert kv.ctx_len == [255, 18]
    k1, v1 = kv.k, kv.v
    for b, (C, p) in enumerate(zip(ctx, paths)):
        for i, n in enumerate(p):
            assert torch.equal(k1[:, b, :, C + i, :], k0[:, b, :, C + n, :])
            assert torch.equal(v1[:, b, :, :, C + i], v0[:, b, :, :, C + n])
        untouched = [s for s in range(512) if not (C <= s < C + len(p))]
        assert torch.equal(k1[:, b, :, untouched, :], k0[:, b, :, untouched, :])
        assert torch.equal(v1[:, b, :, :, untouched], v0[:, b, :, :, untouched])
    mapped = set(kv.table.flatten().tolist())
    spare = [p for p in range(kv.n_pages) if p not in mapped]
    assert torch.equal(kv.k_pool[:, spare], pools[0][:, spare]) and torch.equal(kv.v_pool[:, spare], pools[1][:, spare])


def test_a_page_id_outside_the_pool_is_clamped_not_followed():
    """A bad table entry must not become a stray access: the id is clamped into the pool (the
    results are then wrong, which is the caller's doing; the status word stays clear)."""
    shape = TB.with_(n_layers=1)
    case = make_case(shape, 13, [300], [gen_chain(5)])
    model = device_model(shape, case.seed)
    good = case.run_gpu(0.5, model=model, paged=True)
    kv = good["_kv"]
    kv.table[0, 1] = 10 ** 6                          # far outside the pool
    out = good["_ver"].verify(kv, good["_tok"], case.parents, torch.from_numpy(case.positions).cuda(), 0.5)
    torch.cuda.synchronize()
    assert out["status"].item() == 0 and out["accepted_len"].item() >= 0


def test_rounds_are_the_same_with_paged_caches():
    """The round driver (commits and catch-up included) over paged caches emits what it emits over
    contiguous ones."""
    from paper_2601_23180_amd import TernaryDecoder
    from test_gpu_rounds import mixed_drafts
    shape = SHAPES["tiny"]
    Wp = oracle_weights(shape, 61)
    prompt = gen_context_tokens(shape.vocab, 250, 61).tolist()       # the rounds cross the first page end
    drafts = mixed_drafts(Wp, shape, 61, 12)
    runs = []
    for paged in (False, True):
        dec = TernaryDecoder(device_model(shape, 61), device_model(shape, 62), 512, max_nodes=16, paged=paged)
        dec.start(prompt)
        recs = [dec.round(*drafts(r, dec.seq), 0.35) for r in range(6)]
        runs.append((recs, dec.seq, dec.kv_p.ctx_len, dec.kv_t.ctx_len))
        n = dec.kv_p.ctx_len[0]
        runs[-1] += (dec.kv_p.k[:, 0, :, :n, :].float().cpu(),)
        dec.close()
    assert runs[0][:4] == runs[1][:4]
    assert torch.equal(runs[0][4], runs[1][4])
    assert runs[0][2][0] > 256
