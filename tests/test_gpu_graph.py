"""The hot path under HIP graph capture: the library allocates nothing, never synchronises and uses no
memset, so one step (selection, forward, backward) can be captured once and replayed.  Every replay is
checked against the eager result (bit for bit: the kernels are deterministic), with eager work and
synchronisations between the replays."""
import pytest
import torch

from paper_2602_02108_amd import api
from paper_2602_02108_amd.workloads import WORKLOADS, make_inputs, torch_dtype

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["mid_sparse_bf16", "tiny_sparse"])
def test_captured_step_replays_like_the_eager_step(name):
    w = WORKLOADS[name]
    x = make_inputs(w, "cuda")
    desc = api.make_desc(x["q"], x["k_pool"], w.N, w.sm_scale, torch_dtype(w.grad_dtype))
    dev = x["q"].device
    ws = {op: torch.empty(api.workspace_bytes(desc, w.top_k, op), dtype=torch.uint8, device=dev)
          for op in (api.OP_SCORE_TOPK, api.OP_ATTN_FWD, api.OP_ATTN_BWD)}
    sel = torch.empty((w.Hkv, w.top_k + w.m), dtype=torch.int32, device=dev)
    cnt = torch.empty((w.Hkv,), dtype=torch.int32, device=dev)
    o = torch.empty_like(x["q"])
    lse = torch.empty((w.Hq, w.C), dtype=torch.float32, device=dev)
    dq = torch.empty_like(x["q"])

    def step():
        api.page_score_topk(desc, x["q"], x["k_pool"], x["page_table"], w.top_k, sel, cnt, workspace=ws[api.OP_SCORE_TOPK])
        api.paged_attn_fwd(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], sel, cnt, o, lse, ws[api.OP_ATTN_FWD])
        api.paged_attn_bwd(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], o, lse, x["d_o"], x["dk_pool"],
                           x["dv_pool"], sel, cnt, dq, ws[api.OP_ATTN_BWD])

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (sel, cnt, o, lse, dq, x["dk_pool"], x["dv_pool"])]

    step()                                   # eager (also sets the kernels' attributes before any capture)
    want = snapshot()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        for t in (x["dk_pool"], x["dv_pool"]):
            t.zero_()
        step()                               # warm-up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)

    for r in range(3):
        for t in (sel, cnt, o, lse, dq):     # eager work between the replays: scribble over the outputs
            t.zero_()
        x["dk_pool"].zero_()
        x["dv_pool"].zero_()
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for a, b in zip(got, want):
            assert torch.equal(a, b), f"replay {r} differs from the eager step"


def test_captured_votes_step_replays_like_the_eager_step():
    """The per-query-page path (votes, list maps built on the device, attention over one list per query page)
    under capture: same check as above."""
    w = WORKLOADS["mid_sparse_bf16"]
    top_k = w.top_k
    x = make_inputs(w, "cuda")
    desc = api.make_desc(x["q"], x["k_pool"], w.N, w.sm_scale, torch_dtype(w.grad_dtype))
    dev = x["q"].device
    ws = {op: torch.empty(api.workspace_bytes(desc, top_k, op), dtype=torch.uint8, device=dev)
          for op in (api.OP_VOTE_TOPK, api.OP_ATTN_FWD_QP, api.OP_ATTN_BWD_QP)}
    cache = torch.zeros((w.n, w.Hkv, w.D), dtype=torch.float32, device=dev)
    sel = torch.empty((w.Hkv, w.m, top_k + w.m), dtype=torch.int32, device=dev)
    cnt = torch.empty((w.Hkv, w.m), dtype=torch.int32, device=dev)
    o = torch.empty_like(x["q"])
    lse = torch.empty((w.Hq, w.C), dtype=torch.float32, device=dev)
    dq = torch.empty_like(x["q"])

    def step():
        api.page_means(desc, x["k_pool"], x["page_table"], 0, w.n_past, cache)
        api.page_vote_topk(desc, x["q"], cache, top_k, sel, cnt, workspace=ws[api.OP_VOTE_TOPK])
        api.paged_attn_fwd_qp(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], sel, cnt, o, lse,
                              ws[api.OP_ATTN_FWD_QP])
        api.paged_attn_bwd_qp(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], o, lse, x["d_o"], x["dk_pool"],
                              x["dv_pool"], sel, cnt, dq, ws[api.OP_ATTN_BWD_QP])

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (sel, cnt, o, lse, dq, x["dk_pool"], x["dv_pool"])]

    step()
    want = snapshot()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        for t in (x["dk_pool"], x["dv_pool"]):
            t.zero_()
        step()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for r in range(3):
        for t in (sel, cnt, o, lse, dq, cache):
            t.zero_()
        x["dk_pool"].zero_()
        x["dv_pool"].zero_()
        for buf in ws.values():           # the maps and partial sums of the last replay must not matter
            buf.fill_(0x5a)
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for a, b in zip(got, want):
            assert torch.equal(a, b), f"replay {r} differs from the eager step"


def test_captured_offloaded_step_replays_like_the_eager_step():
    """A whole offloaded step in one graph: selection, staging plan, fetch from pinned host pools, attention on
    the staging pools, gradient write-back into the pinned host pools."""
    w = WORKLOADS["mid_sparse_bf16"]
    x = make_inputs(w, "cuda")
    desc = api.make_desc(x["q"], x["k_pool"], w.N, w.sm_scale, torch_dtype(w.grad_dtype))
    dev = x["q"].device
    gdt = torch_dtype(w.grad_dtype)

    def pinned(t):
        h = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
        h.copy_(t)
        return h

    host_k, host_v = pinned(x["k_pool"]), pinned(x["v_pool"])
    host_dk = torch.zeros(x["k_pool"].shape, dtype=gdt, pin_memory=True)
    host_dv = torch.zeros(x["k_pool"].shape, dtype=gdt, pin_memory=True)
    ws = {op: torch.empty(api.workspace_bytes(desc, w.top_k, op), dtype=torch.uint8, device=dev)
          for op in (api.OP_SCORE_TOPK, api.OP_ATTN_FWD, api.OP_ATTN_BWD)}
    sel = torch.empty((w.Hkv, w.top_k + w.m), dtype=torch.int32, device=dev)
    cnt = torch.empty((w.Hkv,), dtype=torch.int32, device=dev)
    cache = torch.zeros((w.n, w.Hkv, w.D), dtype=torch.float32, device=dev)
    api.page_means(desc, x["k_pool"], x["page_table"], 0, w.n_past, cache)
    cap = api.offload_capacity(desc, sel)
    plan = api.OffloadPlan(desc, cap, dev)
    shape = (cap,) + tuple(x["k_pool"].shape[1:])
    stage_k = torch.zeros(shape, dtype=x["k_pool"].dtype, device=dev)
    stage_v = torch.zeros_like(stage_k)
    stage_dk = torch.zeros(shape, dtype=gdt, device=dev)
    stage_dv = torch.zeros_like(stage_dk)
    o = torch.empty_like(x["q"])
    lse = torch.empty((w.Hq, w.C), dtype=torch.float32, device=dev)
    dq = torch.empty_like(x["q"])

    def step():
        api.page_score_topk_cached(desc, x["q"], cache, w.top_k, sel, cnt, workspace=ws[api.OP_SCORE_TOPK])
        api.offload_plan(desc, sel, cnt, plan=plan)
        api.offload_fetch(desc, host_k, host_v, x["page_table"], plan, stage_k, stage_v, stage_dk, stage_dv)
        api.paged_attn_fwd(desc, x["q"], stage_k, stage_v, plan.stage_table, sel, cnt, o, lse, ws[api.OP_ATTN_FWD])
        api.paged_attn_bwd(desc, x["q"], stage_k, stage_v, plan.stage_table, o, lse, x["d_o"], stage_dk, stage_dv, sel, cnt,
                           dq, ws[api.OP_ATTN_BWD])
        api.offload_writeback(desc, stage_dk, stage_dv, host_dk, host_dv, x["page_table"], plan)

    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in (sel, o, lse, dq, host_dk, host_dv)]
    # the resident path gives the same bits
    res_o, res_lse = api.paged_attn_fwd(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], sel, cnt)
    torch.cuda.synchronize()
    assert torch.equal(res_o, o) and torch.equal(res_lse, lse)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for r in range(3):
        host_dk.zero_()
        host_dv.zero_()
        for t in (sel, o, lse, dq, stage_k, stage_v):
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip((sel, o, lse, dq, host_dk, host_dv), want):
            assert torch.equal(a, b), f"replay {r} differs from the eager step"
