"""GPU parity of the paged-manager steps either side of the attention path: append (bit-exact
pools and page means), selection from cached page means (bit-exact scores and lists), the
local-attention page list and attention over it."""
import numpy as np
import pytest
import torch

import oracle as orc
from paper_2602_02108_amd import api
from paper_2602_02108_amd.workloads import WORKLOADS, Workload, make_inputs, to_numpy, torch_dtype

import parity_util as pu

pytestmark = pytest.mark.gpu

CASES = [WORKLOADS["tiny_sparse"], WORKLOADS["smoke_bf16"], WORKLOADS["mid_sparse_bf16"],
         Workload("bf16_p64_mgr", 8, 2, 128, 64, 192, 64 * 19, 5, "bf16", "bf16", 0.088, extra_phys=3, seed=21)]


def _bits(a):
    a = np.ascontiguousarray(a)
    return a.view(np.uint16) if a.dtype == np.uint16 else a.view(np.uint32)


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_append_and_page_means_are_bit_exact(w):
    x = make_inputs(w, "cuda")
    sh = pu.shape_of(w)
    dt = x["k_pool"].dtype
    gen = torch.Generator(device="cpu").manual_seed(w.seed + 99)
    kc = torch.randn((w.C, w.Hkv, w.D), generator=gen).to(dt).cuda()
    vc = torch.randn((w.C, w.Hkv, w.D), generator=gen).to(dt).cuda()
    desc = api.make_desc(x["q"], x["k_pool"], w.N, w.sm_scale, torch_dtype(w.grad_dtype))
    cache = torch.full((sh.n, w.Hkv, w.D), 7.0, dtype=torch.float32, device="cuda")
    hk, hv, hpt = to_numpy(x["k_pool"]), to_numpy(x["v_pool"]), to_numpy(x["page_table"])
    ok, ov, ocache = orc.kv_append(sh, to_numpy(kc), to_numpy(vc), hpt, hk, hv, cache.cpu().numpy())
    api.kv_append(desc, kc, vc, x["page_table"], x["k_pool"], x["v_pool"], cache)
    torch.cuda.synchronize()
    assert np.array_equal(_bits(to_numpy(x["k_pool"])), _bits(ok)), "K pool differs"
    assert np.array_equal(_bits(to_numpy(x["v_pool"])), _bits(ov)), "V pool differs"
    assert np.array_equal(cache.cpu().numpy().view(np.uint32), ocache.view(np.uint32)), "cached means differ"
    # rebuilding the whole cache from the pool gives the same rows for the appended pages
    cache2 = torch.zeros_like(cache)
    api.page_means(desc, x["k_pool"], x["page_table"], 0, sh.n, cache2)
    torch.cuda.synchronize()
    want = orc.page_means(sh, ok, hpt, 0, sh.n, np.zeros((sh.n, w.Hkv, w.D), np.float32))
    assert np.array_equal(cache2.cpu().numpy().view(np.uint32), want.view(np.uint32))
    assert np.array_equal(cache2.cpu().numpy()[sh.n_past:].view(np.uint32), ocache[sh.n_past:].view(np.uint32))


@pytest.mark.parametrize("name", ["tiny_sparse", "smoke_bf16", "mid_sparse_bf16", "qwen_sparse_256k"])
def test_selection_from_cached_means_is_bit_exact(name):
    w = WORKLOADS[name]
    x = make_inputs(w, "cuda")
    sh = pu.shape_of(w)
    desc = api.make_desc(x["q"], x["k_pool"], w.N, w.sm_scale, torch_dtype(w.grad_dtype))
    cache = torch.zeros((sh.n, w.Hkv, w.D), dtype=torch.float32, device="cuda")
    api.page_means(desc, x["k_pool"], x["page_table"], 0, sh.n_past, cache)
    scores = torch.empty((w.Hkv, max(sh.n_past, 1)), dtype=torch.float32, device="cuda")
    sel, cnt = api.page_score_topk_cached(desc, x["q"], cache, w.top_k, scores_out=scores)
    torch.cuda.synchronize()
    hx = pu.host_inputs(x)
    # oracle: streaming selection (pinned by brute force) == cached selection, and the GPU cache == oracle cache
    osel, ocnt, oscores = pu.oracle_select(w, hx)
    assert np.array_equal(scores[:, :sh.n_past].cpu().numpy().view(np.uint32), oscores.view(np.uint32)), "scores differ"
    assert np.array_equal(cnt.cpu().numpy(), ocnt) and np.array_equal(sel.cpu().numpy(), osel)
    if sh.n_past * w.Hkv * w.D <= (1 << 24):
        ocache = orc.page_means(sh, hx["k_pool"], hx["page_table"], 0, sh.n_past, np.zeros((sh.n, w.Hkv, w.D), np.float32))
        assert np.array_equal(cache.cpu().numpy().view(np.uint32), ocache.view(np.uint32))
        csel, ccnt, cscores = orc.page_score_topk_cached(sh, hx["q"], ocache, w.top_k)
        assert np.array_equal(cscores.view(np.uint32), oscores.view(np.uint32)) and np.array_equal(csel, osel)


@pytest.mark.parametrize("name,window", [("tiny_sparse", 0), ("tiny_sparse", 5), ("tiny_sparse", 1000),
                                         ("mid_sparse_bf16", 3), ("smoke_bf16", 2)])
def test_local_page_list_and_attention_over_it(name, window):
    w = WORKLOADS[name]
    x = make_inputs(w, "cuda")
    sh = pu.shape_of(w)
    desc = api.make_desc(x["q"], x["k_pool"], w.N, w.sm_scale, torch_dtype(w.grad_dtype))
    sel, cnt = api.local_page_list(desc, window, "cuda")
    torch.cuda.synchronize()
    osel, ocnt = orc.local_page_list(sh, window)
    assert np.array_equal(sel.cpu().numpy(), osel) and np.array_equal(cnt.cpu().numpy(), ocnt)
    hx = pu.host_inputs(x)
    res = pu.gpu_fwd_bwd(w, x, sel, cnt)
    ref = pu.oracle_fwd_bwd(w, hx, osel, ocnt)
    dt = w.dtype
    pu.check("O", pu.f32(res["o"]), ref["o"], dt)
    pu.check("LSE", pu.f32(res["lse"]), ref["lse"], "f32" if dt == "f32" else "bf16")
    pu.check("dQ", pu.f32(res["dq"]), ref["dq"], dt)
    pu.check("dK", pu.f32(res["dk_pool"]), ref["dk_pool"], dt)
    pu.check("dV", pu.f32(res["dv_pool"]), ref["dv_pool"], dt)
