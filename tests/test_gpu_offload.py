"""GPU parity of the offload steps (paper Sec. 4.3): the K / V pools and the gradient pools sit in pinned
host memory, the pages in the lists are fetched into device staging pools by kernels that read the host
memory directly, attention runs on the staging pools, the gradients of the fetched pages are added back
to the host pools.  Data movement is compared bit for bit with the oracle; the attention over staged
pages must reproduce the attention over a resident pool bit for bit, and match the oracle."""
import numpy as np
import pytest
import torch

from paper_2602_02108_amd import api
from paper_2602_02108_amd.workloads import WORKLOADS, Workload, make_inputs, to_numpy, torch_dtype

import oracle as orc
import parity_util as pu

pytestmark = pytest.mark.gpu

CASES = [
    WORKLOADS["tiny_sparse"],                                    # fp32, shape-generic kernels
    WORKLOADS["mid_sparse_bf16"],                                # bf16 MFMA kernels, fp32 gradient pool
    Workload("off_bf16grad", 8, 2, 128, 128, 256, 128 * 14, 3, "bf16", "bf16", 0.0884, extra_phys=2, boost_frac=0.2,
             seed=51),
]


def _bits(a):
    a = np.ascontiguousarray(a)
    return a.view(np.uint16) if a.dtype.itemsize == 2 else a.view(np.uint32)


def _pinned(t):
    h = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
    h.copy_(t)
    return h


def _setup(w):
    x = make_inputs(w, "cuda")
    desc = api.make_desc(x["q"], x["k_pool"], w.N, w.sm_scale, torch_dtype(w.grad_dtype))
    sel, cnt, _ = pu.gpu_select(w, x)
    torch.cuda.synchronize()
    return x, desc, sel, cnt


def _check_movement(w, x, desc, sel, cnt):
    """plan / fetch / write-back against the oracle, bit for bit, for lists of either shape."""
    hx = pu.host_inputs(x)
    sh = pu.shape_of(w)
    hsel, hcnt = sel.cpu().numpy(), cnt.cpu().numpy()
    plan = api.offload_plan(desc, sel, cnt)
    torch.cuda.synchronize()
    otable, oslots, omask = orc.offload_plan(sh, hsel, hcnt)
    ns = int(plan.n_slots.item())
    assert ns == len(oslots) <= plan.capacity
    assert np.array_equal(plan.stage_table.cpu().numpy(), otable)
    assert np.array_equal(plan.slot_pages.cpu().numpy()[:ns], oslots)
    assert np.array_equal(plan.head_mask.cpu().numpy().view(np.uint32), omask)

    cap = plan.capacity
    host_k, host_v = _pinned(x["k_pool"]), _pinned(x["v_pool"])
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    junk = lambda dt: (torch.randn((cap,) + tuple(x["k_pool"].shape[1:]), generator=g, device="cuda")).to(dt)
    stage_k, stage_v = junk(x["k_pool"].dtype), junk(x["k_pool"].dtype)
    gdt = torch_dtype(w.grad_dtype)
    stage_dk, stage_dv = junk(gdt), junk(gdt)
    before = [t.clone() for t in (stage_k, stage_v, stage_dk, stage_dv)]
    api.offload_fetch(desc, host_k, host_v, x["page_table"], plan, stage_k, stage_v, stage_dk, stage_dv)
    torch.cuda.synchronize()
    ok, ov = orc.offload_fetch(sh, hx["k_pool"], hx["v_pool"], hx["page_table"], oslots, omask,
                               to_numpy(before[0]), to_numpy(before[1]))
    assert np.array_equal(_bits(to_numpy(stage_k)), _bits(ok)) and np.array_equal(_bits(to_numpy(stage_v)), _bits(ov))
    # gradient staging: held tiles zeroed, the rest untouched
    held = np.zeros((cap, w.Hkv), bool)
    for s_, l in enumerate(oslots):
        for gg in range(w.Hkv):
            held[s_, gg] = (int(omask[l]) >> gg) & 1
    for got, was in ((stage_dk, before[2]), (stage_dv, before[3])):
        got, was = got.float().cpu().numpy(), was.float().cpu().numpy()
        assert not got[held].any() and np.array_equal(got[~held], was[~held])

    # write-back: host += staged gradients (seeded values on both sides)
    stage_dk.copy_(before[2])
    stage_dv.copy_(before[3])
    h0k = torch.randn(x["k_pool"].shape, generator=torch.Generator().manual_seed(8)).to(gdt)
    h0v = torch.randn(x["k_pool"].shape, generator=torch.Generator().manual_seed(9)).to(gdt)
    host_dk, host_dv = _pinned(h0k), _pinned(h0v)
    api.offload_writeback(desc, stage_dk, stage_dv, host_dk, host_dv, x["page_table"], plan)
    torch.cuda.synchronize()
    wk, wv = orc.offload_writeback(sh, before[2].float().cpu().numpy()[:ns], before[3].float().cpu().numpy()[:ns],
                                   h0k.float().numpy(), h0v.float().numpy(), hx["page_table"], oslots, omask)
    if w.grad_dtype == "bf16":  # the sum is rounded to the pool's dtype
        wk = torch.from_numpy(wk).to(torch.bfloat16).float().numpy()
        wv = torch.from_numpy(wv).to(torch.bfloat16).float().numpy()
    assert np.array_equal(host_dk.float().numpy(), wk) and np.array_equal(host_dv.float().numpy(), wv)


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_plan_fetch_writeback_move_the_right_tiles(w):
    x, desc, sel, cnt = _setup(w)
    _check_movement(w, x, desc, sel, cnt)


def test_movement_with_one_list_per_query_page():
    from test_gpu_qp_attention import rand_qp_lists
    w = CASES[1]
    x, desc, _, _ = _setup(w)
    sel, cnt = rand_qp_lists(w, 4, 61, popular=2)
    _check_movement(w, x, desc, torch.as_tensor(sel, device="cuda"), torch.as_tensor(cnt, device="cuda"))


def _offloaded_pass(w, x, desc, sel, cnt, qp):
    """Pools in pinned host memory, staging pools poisoned with NaN, fetch and write-back on a stream of their own."""
    host_k, host_v = _pinned(x["k_pool"]), _pinned(x["v_pool"])
    gdt = torch_dtype(w.grad_dtype)
    host_dk = torch.zeros(x["k_pool"].shape, dtype=gdt, pin_memory=True)
    host_dv = torch.zeros(x["k_pool"].shape, dtype=gdt, pin_memory=True)
    cap = api.offload_capacity(desc, sel)
    shape = (cap,) + tuple(x["k_pool"].shape[1:])
    stage_k = torch.full(shape, float("nan"), dtype=x["k_pool"].dtype, device="cuda")
    stage_v = torch.full(shape, float("nan"), dtype=x["k_pool"].dtype, device="cuda")
    stage_dk = torch.full(shape, float("nan"), dtype=gdt, device="cuda")
    stage_dv = torch.full(shape, float("nan"), dtype=gdt, device="cuda")
    copy_stream = torch.cuda.Stream()
    main = torch.cuda.current_stream()
    plan = api.offload_plan(desc, sel, cnt)
    planned = torch.cuda.Event()
    planned.record(main)
    copy_stream.wait_event(planned)
    api.offload_fetch(desc, host_k, host_v, x["page_table"], plan, stage_k, stage_v, stage_dk, stage_dv, stream=copy_stream)
    fetched = torch.cuda.Event()
    fetched.record(copy_stream)
    main.wait_event(fetched)
    staged_pt = plan.stage_table.clamp(min=0)
    fwd = api.paged_attn_fwd_qp if qp else api.paged_attn_fwd
    bwd = api.paged_attn_bwd_qp if qp else api.paged_attn_bwd
    o, lse = fwd(desc, x["q"], stage_k, stage_v, staged_pt, sel, cnt)
    dq = bwd(desc, x["q"], stage_k, stage_v, staged_pt, o, lse, x["d_o"], stage_dk, stage_dv, sel, cnt)
    done = torch.cuda.Event()
    done.record(main)
    copy_stream.wait_event(done)
    api.offload_writeback(desc, stage_dk, stage_dv, host_dk, host_dv, x["page_table"], plan, stream=copy_stream)
    torch.cuda.synchronize()
    return o, lse, dq, host_dk, host_dv


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_attention_over_staged_pages_equals_the_resident_pool(w):
    x, desc, sel, cnt = _setup(w)
    hx = pu.host_inputs(x)
    res = pu.gpu_fwd_bwd(w, x, sel, cnt)
    res = {k: v.clone() for k, v in res.items()}
    o, lse, dq, host_dk, host_dv = _offloaded_pass(w, x, desc, sel, cnt, qp=False)
    assert torch.equal(o, res["o"]) and torch.equal(lse, res["lse"]) and torch.equal(dq, res["dq"])
    assert torch.equal(host_dk, res["dk_pool"].cpu()) and torch.equal(host_dv, res["dv_pool"].cpu())
    # and against the oracle
    osel, ocnt, _ = pu.oracle_select(w, hx)
    ref = pu.oracle_fwd_bwd(w, hx, osel, ocnt)
    gd = w.dtype if w.grad_dtype == "f32" else "bf16"
    pu.check("O", pu.f32(o), ref["o"], w.dtype)
    pu.check("dQ", pu.f32(dq), ref["dq"], w.dtype)
    pu.check("dK (host pool)", host_dk.float().numpy(), ref["dk_pool"], gd)
    pu.check("dV (host pool)", host_dv.float().numpy(), ref["dv_pool"], gd)


def test_offloaded_pass_with_one_list_per_query_page():
    """Votes-style lists: the offloaded pass reproduces the resident one bit for bit and matches the oracle."""
    from test_gpu_qp_attention import rand_qp_lists, gpu_fwd_bwd_qp
    w = CASES[1]
    x, desc, _, _ = _setup(w)
    hx = pu.host_inputs(x)
    sel, cnt = rand_qp_lists(w, 4, 62, popular=2)
    dsel, dcnt = torch.as_tensor(sel, device="cuda"), torch.as_tensor(cnt, device="cuda")
    res = gpu_fwd_bwd_qp(w, x, sel, cnt)
    res = {k: v.clone() for k, v in res.items()}
    o, lse, dq, host_dk, host_dv = _offloaded_pass(w, x, desc, dsel, dcnt, qp=True)
    assert torch.equal(o, res["o"]) and torch.equal(lse, res["lse"]) and torch.equal(dq, res["dq"])
    assert torch.equal(host_dk, res["dk_pool"].cpu()) and torch.equal(host_dv, res["dv_pool"].cpu())
    ref = orc.attn_fwd_bwd(pu.shape_of(w), hx["q"], hx["k_pool"], hx["v_pool"], hx["page_table"], hx["d_o"], sel, cnt,
                           prec="f32")
    pu.check("O", pu.f32(o), ref["o"], w.dtype)
    pu.check("dK (host pool)", host_dk.float().numpy(), ref["dk_pool"], w.dtype)


def test_host_pools_that_the_device_cannot_address_are_refused():
    w = CASES[0]
    x, desc, sel, cnt = _setup(w)
    plan = api.offload_plan(desc, sel, cnt)
    stage = torch.zeros((plan.capacity,) + tuple(x["k_pool"].shape[1:]), dtype=x["k_pool"].dtype, device="cuda")
    pageable = x["k_pool"].cpu()   # ordinary (pageable) host memory
    with pytest.raises(api.OombError):
        api.offload_fetch(desc, pageable, pageable, x["page_table"], plan, stage, stage.clone())
    torch.cuda.synchronize()
