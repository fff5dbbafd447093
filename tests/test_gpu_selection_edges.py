"""GPU parity of the page selection (Sec. 4.2 top-K) on inputs built to tie: the page means are copies of a
handful of distinct rows, so that scores are equal bit for bit in large groups and the cut of the top-k falls
inside a group (ties go to the lower logical id), with all-zero rows of either sign whose scores are +0 and -0
(equal under the comparison).  List lengths cover every instantiation of the register-resident selection
kernel and the kernel for longer lists.  The means are handed over through the cached-means entry point (the
selection kernel is the same as behind the streaming scorer, which a second test runs on tied pages)."""
import numpy as np
import pytest
import torch

from paper_2602_02108_amd import api

import oracle as orc
from oracle import Shape

pytestmark = pytest.mark.gpu

HQ, HKV, D, P, C = 4, 2, 64, 16, 32
M = C // P


def _query(g):
    return torch.randn((C, HQ, D), generator=g, device="cuda").abs() + 0.1   # positive: x * (-0) = -0


def _check(desc, sh, q, n_past, run_gpu, run_oracle):
    for top_k in sorted({0, 1, 7, max(n_past // 3, 1), n_past, n_past + 5}):
        scores = torch.empty((HKV, max(n_past, 1)), dtype=torch.float32, device="cuda")
        sel, cnt = run_gpu(top_k, scores)
        torch.cuda.synchronize()
        osel, ocnt, oscores = run_oracle(top_k)
        assert np.array_equal(scores[:, :n_past].cpu().numpy().view(np.uint32), oscores.view(np.uint32)), (n_past, top_k)
        assert np.array_equal(cnt.cpu().numpy(), ocnt), (n_past, top_k)
        assert np.array_equal(sel.cpu().numpy(), osel), (n_past, top_k)
    return oscores


@pytest.mark.parametrize("n_past", [0, 1, 5, 1023, 1024, 1025, 2049, 4100, 8191, 12289, 16385, 24577, 32768, 32769, 40000])
def test_selection_with_tied_scores(n_past):
    g = torch.Generator(device="cuda")
    g.manual_seed(1000 + n_past)
    n = n_past + M
    base = torch.randn((7, HKV, D), generator=g, device="cuda")
    base[5] = 0.0
    base[6] = -0.0
    kbar = base[torch.randint(0, 7, (n,), generator=g, device="cuda")].contiguous()
    q = _query(g)
    k_shape = torch.empty((1, HKV, P, D), device="cuda").expand(n, HKV, P, D)   # shape / strides for the descriptor only
    desc = api.make_desc(q, k_shape, n * P, 0.125)
    desc.pool_page_stride = HKV * P * D
    sh = Shape(HQ, HKV, D, P, C, n * P, 0.125)
    hq, hkb = q.cpu().numpy(), kbar.cpu().numpy()
    oscores = _check(desc, sh, q, n_past,
                     lambda k, sc: api.page_score_topk_cached(desc, q, kbar, k, scores_out=sc),
                     lambda k: orc.page_score_topk_cached(sh, hq, hkb, k))
    if n_past >= 1024:
        # the inputs do what they were built for: few distinct scores, zeros of both signs among them
        vals, counts = np.unique(oscores[0].view(np.uint32), return_counts=True)
        assert len(vals) <= 7 and counts.max() >= n_past // 10
        assert 0x00000000 in vals and 0x80000000 in vals


@pytest.mark.parametrize("n_past", [777, 9000])
def test_streaming_scorer_on_tied_pages(n_past):
    g = torch.Generator(device="cuda")
    g.manual_seed(2000 + n_past)
    n = n_past + M
    base = torch.randn((6, HKV, P, D), generator=g, device="cuda")
    base[5] = 0.0
    page_table = torch.randperm(n, generator=g, device="cuda").to(torch.int32)
    k_pool = torch.empty((n, HKV, P, D), device="cuda")
    k_pool[page_table.long()] = base[torch.randint(0, 6, (n,), generator=g, device="cuda")]
    q = _query(g)
    desc = api.make_desc(q, k_pool, n * P, 0.125)
    sh = Shape(HQ, HKV, D, P, C, n * P, 0.125)
    hq, hk, hpt = q.cpu().numpy(), k_pool.cpu().numpy(), page_table.cpu().numpy()
    _check(desc, sh, q, n_past,
           lambda k, sc: api.page_score_topk(desc, q, k_pool, page_table, k, scores_out=sc),
           lambda k: orc.page_score_topk(sh, hq, hk, hpt, k))
