"""GPU test of oomb_page_score_topk_noalloc (the entry point for callers that cannot allocate): same lists,
counts and scores, bit for bit, as oomb_page_score_topk, on two calls in a row that share the built-in
scratch array, the second with a smaller input."""
import pytest
import torch

from paper_2602_02108_amd import api
from paper_2602_02108_amd.workloads import WORKLOADS, make_inputs, torch_dtype

pytestmark = pytest.mark.gpu


def _both(w, with_scores):
    x = make_inputs(w, "cuda", zero_grad_pools=False)
    dev = x["q"].device
    desc = api.make_desc(x["q"], x["k_pool"], w.N, w.sm_scale, torch_dtype(w.grad_dtype))
    want_sel, want_cnt = api.page_score_topk(desc, x["q"], x["k_pool"], x["page_table"], w.top_k)
    want_scores = torch.empty((w.Hkv, w.n_past), dtype=torch.float32, device=dev)
    api.page_score_topk(desc, x["q"], x["k_pool"], x["page_table"], w.top_k, scores_out=want_scores)
    sel = torch.full((w.Hkv, w.top_k + w.m), -7, dtype=torch.int32, device=dev)
    cnt = torch.full((w.Hkv,), -7, dtype=torch.int32, device=dev)
    scores = torch.full((w.Hkv, w.n_past), float("nan"), dtype=torch.float32, device=dev) if with_scores else None
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated(dev)
    api.page_score_topk_noalloc(desc, x["q"], x["k_pool"], x["page_table"], w.top_k, sel, cnt, scores)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated(dev) == before
    assert torch.equal(cnt, want_cnt), (w.name, cnt.tolist(), want_cnt.tolist())
    assert torch.equal(sel, want_sel), w.name
    if with_scores:
        assert torch.equal(scores.view(torch.int32), want_scores.view(torch.int32)), w.name


def test_noalloc_scoring_matches_workspace_scoring_on_consecutive_calls():
    # large first (its scores stay behind in the shared scratch), then a smaller shape, then fp32 tensors
    _both(WORKLOADS["qwen_sparse_256k"], with_scores=False)
    _both(WORKLOADS["mid_sparse_bf16"], with_scores=False)
    _both(WORKLOADS["mid_sparse_bf16"], with_scores=True)
    _both(WORKLOADS["tiny_sparse"], with_scores=False)
    _both(WORKLOADS["qwen_sparse_256k"], with_scores=True)
