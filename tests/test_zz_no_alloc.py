"""trispec_sample_decide_static — the entry point for callers that cannot allocate device memory —
against trispec_sample_decide on the same inputs: the two run the same kernels, one on the
library's own scratch area, one on a caller buffer, so every output must be identical.  Two calls
in a row, the second with a smaller input (the area keeps the first call's contents), then the
size limit."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import CRIT_MARGIN, CRIT_TOP1, RESAMPLE_DIRECT, RESAMPLE_RESIDUAL
from paper_2601_23180_amd import SampleDecider
from paper_2601_23180_amd import binding as B
from workloads import gen_draft_distributions, gen_uniforms

pytestmark = pytest.mark.gpu


def _inputs(seed, batch, n_nodes, vocab, T):
    rng = np.random.default_rng(seed)
    logits = (rng.standard_normal((batch, n_nodes, vocab)) * 3.0).astype(np.float32)
    pd, tk = zip(*[gen_draft_distributions(logits[b], T, seed * 10 + b) for b in range(batch)])
    ua, us = gen_uniforms(seed, batch, n_nodes)
    dev = lambda x, dt: torch.from_numpy(np.ascontiguousarray(x)).to(dt).cuda()
    return (dev(logits, torch.float32), dev(np.stack(tk), torch.int32), dev(np.stack(pd), torch.float32),
            dev(ua, torch.float32), dev(us, torch.float32))


def _both(seed, batch, n_nodes, vocab, T, lam, crit, n_forced, resample):
    args = _inputs(seed, batch, n_nodes, vocab, T)
    res = []
    for static in (False, True):
        dec = SampleDecider(batch, n_nodes, vocab, static_scratch=static)
        for t in dec.out.values():
            t.fill_(-7)
        out = dec.decide(*args, T, lam, crit, n_forced, resample)
        torch.cuda.synchronize()
        res.append({k: v.cpu().numpy().copy() for k, v in out.items()})
    return res


def test_static_scratch_entry_point_equals_the_caller_scratch_one():
    # first a large call, then a smaller one on the same (now dirty) area, then a large one again
    cases = [(31, 8, 9, 151936, 0.8, 0.02, CRIT_MARGIN, 1, RESAMPLE_RESIDUAL),
             (32, 2, 5, 4099, 1.3, 0.0, CRIT_TOP1, 2, RESAMPLE_DIRECT),
             (33, 1, 1, 3, 1.0, 0.0, CRIT_MARGIN, 1, RESAMPLE_RESIDUAL),
             (34, 4, 9, 50257, 0.6, 0.3, CRIT_TOP1, 1, RESAMPLE_RESIDUAL)]
    drew = 0
    for c in cases:
        ref, got = _both(*c)
        for k in ref:
            assert np.array_equal(ref[k], got[k]), (c, k)
        assert ref["status"][0] == 0
        drew += int((ref["token"] >= 0).sum())
    assert drew > 0   # the comparison covered sampled tokens, not only escalations


def test_static_scratch_refuses_what_does_not_fit():
    lib = B.lib()
    n = C.c_size_t()
    # 256 rows over a 4 M-token vocabulary: far beyond the library's area
    assert lib.trispec_sample_scratch_bytes(8, 32, 4096 * 1024, C.byref(n)) == 0
    assert n.value > (1 << 20)
    one = torch.zeros(1, dtype=torch.float32, device="cuda")
    opts = B.SampleOpts(1.0, RESAMPLE_RESIDUAL, CRIT_MARGIN, 1, one.data_ptr(), one.data_ptr(), one.data_ptr(),
                        None, 0, None)
    out = B.VerifyOut()
    rc = lib.trispec_sample_decide_static(one.data_ptr(), one.data_ptr(), 8, 32, 4096 * 1024, C.c_float(0.0),
                                          C.byref(opts), C.byref(out))
    assert rc == -7   # TRISPEC_EWORKSPACE, before anything is enqueued
    torch.cuda.synchronize()
