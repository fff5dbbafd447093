"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py
times.  The oracle cannot run these whole, so: page selection is compared in full
(bit-exact), O / LSE / dQ on sampled query rows, dK / dV on sampled (KV head, page)
units where the oracle can afford the row statistics of a whole head group, and
and additionally through identities that hold at any size."""
import numpy as np
import pytest
import torch

import oracle as orc
from paper_2602_02108_amd import api
from paper_2602_02108_amd.workloads import WORKLOADS, make_inputs, to_numpy, torch_dtype

import parity_util as pu

pytestmark = pytest.mark.gpu


def _sample_rows(w, n_rand, seed):
    rng = np.random.default_rng(seed)
    rows = {(0, 0), (w.Hq - 1, w.C - 1), (0, w.C - 1), (w.Hq - 1, 0)}
    for i in (w.P - 1, w.P, w.C // 2 - 1, w.C // 2, w.C - w.P, 31, 32):   # page and block boundaries
        for h in (0, w.G - 1, w.G, w.Hq - 1):
            rows.add((h, i))
    while len(rows) < n_rand:
        rows.add((int(rng.integers(w.Hq)), int(rng.integers(w.C))))
    return np.array(sorted(rows), dtype=np.int32)


def _run_gpu(w, x):
    sel = cnt = None
    if w.top_k is not None:
        sel, cnt, scores = pu.gpu_select(w, x)
    else:
        scores = None
    with pu.kernels_ran():   # bf16, P = D = 128: the matrix-core kernels, not the generic ones
        res = pu.gpu_fwd_bwd(w, x, sel, cnt)
    return sel, cnt, scores, res


def _check_rows(w, hx, res, osel, ocnt, rows, lse_full=None, delta_full=None):
    sh = pu.shape_of(w)
    o_r, lse_r = orc.attn_fwd(sh, hx["q"], hx["k_pool"], hx["v_pool"], hx["page_table"], osel, ocnt, rows=rows)
    o_gpu = pu.f32(res["o"])[rows[:, 1], rows[:, 0]]
    lse_gpu = pu.f32(res["lse"])[rows[:, 0], rows[:, 1]]
    pu.check("O (sampled rows)", o_gpu, o_r, w.dtype)
    pu.check("LSE (sampled rows)", lse_gpu, lse_r, "bf16")
    # Delta for the sampled rows from the oracle's own O
    d_o = torch.from_numpy(hx["d_o"].view(np.int16)).view(torch.bfloat16).float().numpy()
    lse = np.zeros((w.Hq, w.C), dtype=np.float32)
    dl = np.zeros((w.Hq, w.C), dtype=np.float32)
    lse[rows[:, 0], rows[:, 1]] = lse_r
    dl[rows[:, 0], rows[:, 1]] = (d_o[rows[:, 1], rows[:, 0]] * o_r).sum(axis=1)
    dq_r = orc.attn_bwd_dq(sh, hx["q"], hx["k_pool"], hx["v_pool"], hx["page_table"], lse, dl, hx["d_o"], osel, ocnt,
                           rows=rows)
    pu.check("dQ (sampled rows)", pu.f32(res["dq"])[rows[:, 1], rows[:, 0]], dq_r, w.dtype)


def _oracle_row_stats(w, hx, osel, ocnt, g):
    """LSE and Delta (oracle, from the oracle's own O) of every row of KV head g's query heads, as [Hq][C]
    arrays that are zero elsewhere: what the oracle's dK / dV of a page of that head needs."""
    sh = pu.shape_of(w)
    heads = np.arange(g * w.G, (g + 1) * w.G)
    rows = np.array([(h, i) for h in heads for i in range(w.C)], dtype=np.int32)
    o_r, lse_r = orc.attn_fwd(sh, hx["q"], hx["k_pool"], hx["v_pool"], hx["page_table"], osel, ocnt, rows=rows)
    d_o = torch.from_numpy(hx["d_o"].view(np.int16)).view(torch.bfloat16).float().numpy()
    lse = np.zeros((w.Hq, w.C), dtype=np.float32)
    dl = np.zeros((w.Hq, w.C), dtype=np.float32)
    lse[rows[:, 0], rows[:, 1]] = lse_r
    dl[rows[:, 0], rows[:, 1]] = (d_o[rows[:, 1], rows[:, 0]] * o_r).sum(axis=1)
    return lse, dl


def _oracle_units(w, hx, osel, ocnt, g, pages, dk, dv):
    """Adds the oracle's dK / dV of the given logical pages of KV head g to dk / dv (fp32 arrays of the pools'
    shape; numpy allocates them lazily, so only the touched pages take memory)."""
    lse, dl = _oracle_row_stats(w, hx, osel, ocnt, g)
    units = np.array([(g, int(l)) for l in pages], dtype=np.int32)
    orc.attn_bwd_dkv(pu.shape_of(w), hx["q"], hx["k_pool"], hx["v_pool"], hx["page_table"], lse, dl, hx["d_o"], dk, dv,
                     osel, ocnt, units=units)


def _compare_units(hx, res, g, pages, dk, dv):
    phys = hx["page_table"][np.asarray(pages)]
    idx = torch.as_tensor(phys, device=res["dk_pool"].device).long()
    pu.check(f"dK (sampled pages, KV head {g})", pu.f32(res["dk_pool"][idx, g]), dk[phys, g], "bf16")
    pu.check(f"dV (sampled pages, KV head {g})", pu.f32(res["dv_pool"][idx, g]), dv[phys, g], "bf16")


def _unit_pages(w, osel, ocnt, g):
    """Eight pages of KV head g: five past pages spread over the list, the first / a middle / the last local
    page (every local page holds the causal diagonal of its own query rows)."""
    if osel is None:   # dense: every page is listed
        lst = np.arange(w.n)
        k = w.n_past
    else:
        lst = osel[g][:ocnt[g]]
        k = int(ocnt[g]) - w.m
    past = [int(lst[j]) for j in sorted({0, k // 4, k // 2, 3 * k // 4, k - 1})] if k > 0 else []
    local = [int(lst[k]), int(lst[k + w.m // 2]), int(lst[k + w.m - 1])]
    return past + local


def _check_pages(w, hx, res, osel, ocnt, g, pages):
    """dK / dV of the given logical pages of KV head g, element by element."""
    dk = np.zeros(hx["k_pool"].shape, dtype=np.float32)
    dv = np.zeros(hx["k_pool"].shape, dtype=np.float32)
    _oracle_units(w, hx, osel, ocnt, g, pages, dk, dv)
    _compare_units(hx, res, g, pages, dk, dv)


def _check_units(w, hx, res, osel, ocnt, heads):
    """dK / dV of sampled (KV head, page) units, element by element.  The KV heads of a call run on different
    XCD pairs of the device, so more than one is sampled."""
    for g in heads:
        _check_pages(w, hx, res, osel, ocnt, g, _unit_pages(w, osel, ocnt, g))


def _check_identities(w, x, res):
    """<dV, V> = sum <dO, O> and <dK, K> = <dQ, Q> per KV head group (pools started at zero)."""
    for g in range(w.Hkv):
        hs = slice(g * w.G, (g + 1) * w.G)
        lhs_v = (res["dv_pool"][:, g].double() * x["v_pool"][:, g].double()).sum().item()
        rhs_v = (x["d_o"][:, hs].double() * res["o"][:, hs].double()).sum().item()
        lhs_k = (res["dk_pool"][:, g].double() * x["k_pool"][:, g].double()).sum().item()
        rhs_k = (res["dq"][:, hs].double() * x["q"][:, hs].double()).sum().item()
        # both sides are sums of ~1e8 bf16-rounded products: compare relative to the mass of the terms
        mass_v = (x["d_o"][:, hs].double().abs() * res["o"][:, hs].double().abs()).sum().item()
        mass_k = (res["dq"][:, hs].double().abs() * x["q"][:, hs].double().abs()).sum().item()
        assert abs(lhs_v - rhs_v) <= 5e-3 * mass_v, (g, lhs_v, rhs_v, mass_v)
        assert abs(lhs_k - rhs_k) <= 5e-3 * mass_k, (g, lhs_k, rhs_k, mass_k)


def _untouched(w, x, res, osel, ocnt, pt):
    for g in range(w.Hkv):
        pages = np.arange(w.n) if osel is None else osel[g][:ocnt[g]]
        untouched = np.setdiff1d(np.arange(w.n_phys), pt[pages])
        if len(untouched):
            idx = torch.as_tensor(untouched, device=res["dk_pool"].device)
            assert not res["dk_pool"][idx, g].any() and not res["dv_pool"][idx, g].any()


@pytest.mark.parametrize("name", ["qwen_sparse_256k", "qwen_sparse_1m"])
def test_sparse_full_size(name):
    w = WORKLOADS[name]
    x = make_inputs(w, "cuda")
    hx = pu.host_inputs(x)
    sel, cnt, scores, res = _run_gpu(w, x)
    osel, ocnt, oscores = pu.oracle_select(w, hx)
    assert np.array_equal(scores.cpu().numpy().view(np.uint32), oscores.view(np.uint32)), "scores differ"
    assert np.array_equal(cnt.cpu().numpy(), ocnt) and np.array_equal(sel.cpu().numpy(), osel)
    # the boosted pages must show up in the selection of the heads whose pooled query points their way
    boosted = set(x["boosted"].cpu().numpy().tolist())
    hit = [len(boosted & set(osel[g][:w.top_k].tolist())) for g in range(w.Hkv)]
    assert max(hit) >= min(len(boosted), w.top_k) * 0.9, hit
    _check_rows(w, hx, res, osel, ocnt, _sample_rows(w, 256, 1))
    _check_units(w, hx, res, osel, ocnt, heads=(1, 2))
    _check_identities(w, x, res)
    _untouched(w, x, res, osel, ocnt, hx["page_table"])


def test_dense_full_size():
    w = WORKLOADS["qwen_dense_64k"]
    x = make_inputs(w, "cuda")
    hx = pu.host_inputs(x)
    _, _, _, res = _run_gpu(w, x)
    _check_rows(w, hx, res, None, None, _sample_rows(w, 96, 2))
    # the only full-size call whose dK / dV workgroups own whole pages and update the pool directly
    _check_units(w, hx, res, None, None, heads=(0, 3))
    _check_identities(w, x, res)


def test_stress_4m_history():
    """4M-token history, chunk 8192, top-k 256, bf16 gradient pool: selection in full, sampled rows, identities."""
    w = WORKLOADS["qwen_sparse_4m"]
    free, _ = torch.cuda.mem_get_info()
    if free < 40 * 2**30:
        pytest.skip("needs ~40 GiB of free HBM")
    x = make_inputs(w, "cuda")
    hx = pu.host_inputs(x)
    sel, cnt, scores, res = _run_gpu(w, x)
    osel, ocnt, oscores = pu.oracle_select(w, hx)
    assert np.array_equal(scores.cpu().numpy().view(np.uint32), oscores.view(np.uint32)), "scores differ"
    assert np.array_equal(cnt.cpu().numpy(), ocnt) and np.array_equal(sel.cpu().numpy(), osel)
    _check_rows(w, hx, res, osel, ocnt, _sample_rows(w, 64, 3))
    # bf16 gradient pool, pages cut into two row slices
    _check_units(w, hx, res, osel, ocnt, heads=(0, 2))
    _check_identities(w, x, res)
    _untouched(w, x, res, osel, ocnt, hx["page_table"])


def _run_sequence(w, x, after_step=None):
    """The 16 calls bench.py times: history growing by one chunk per call, workspaces and outputs allocated once
    for the longest history, gradient pools persisting.  Returns the outputs of the last call and the lists of
    every call (host copies)."""
    dev = x["q"].device
    steps = w.extra_phys // w.m + 1
    assert steps == 16
    gdt = torch_dtype(w.grad_dtype)
    descs = [api.make_desc(x["q"], x["k_pool"], w.N + s * w.C, w.sm_scale, gdt) for s in range(steps)]
    ws = {op: torch.empty(api.workspace_bytes(descs[-1], w.top_k, op), dtype=torch.uint8, device=dev)
          for op in (api.OP_SCORE_TOPK, api.OP_ATTN_FWD, api.OP_ATTN_BWD)}
    sel = torch.empty((w.Hkv, w.top_k + w.m), dtype=torch.int32, device=dev)
    cnt = torch.empty((w.Hkv,), dtype=torch.int32, device=dev)
    o = torch.empty_like(x["q"])
    lse = torch.empty((w.Hq, w.C), dtype=torch.float32, device=dev)
    dq = torch.empty_like(x["q"])
    lists = []
    for s, desc in enumerate(descs):
        api.page_score_topk(desc, x["q"], x["k_pool"], x["page_table"], w.top_k, sel, cnt, workspace=ws[api.OP_SCORE_TOPK])
        api.paged_attn_fwd(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], sel, cnt, o, lse, ws[api.OP_ATTN_FWD])
        api.paged_attn_bwd(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], o, lse, x["d_o"], x["dk_pool"],
                           x["dv_pool"], sel, cnt, dq, ws[api.OP_ATTN_BWD])
        if after_step is not None:
            after_step(s, o, dq)
        lists.append((sel.cpu().numpy().copy(), cnt.cpu().numpy().copy()))
    torch.cuda.synchronize()
    return dict(o=o, lse=lse, dq=dq, dk_pool=x["dk_pool"], dv_pool=x["dv_pool"]), lists


def test_benchmark_sequence_of_16_chunks():
    """The sequence bench.py times.  Checked: the last (longest) call against the oracle -- selection in full,
    sampled rows -- and the pools after all 16 calls through the identities <dV, V> = sum over calls <dO, O> and
    <dK, K> = sum <dQ, Q>, which hold for the accumulated gradients (test_sequence_accumulated_units compares
    accumulated pages with the oracle element by element)."""
    w = WORKLOADS["qwen_sparse_1m"]
    x = make_inputs(w, "cuda")
    hx = pu.host_inputs(x)
    dev = x["q"].device
    rhs_v = torch.zeros(w.Hkv, dtype=torch.float64, device=dev)
    rhs_k = torch.zeros(w.Hkv, dtype=torch.float64, device=dev)
    mass_v = torch.zeros(w.Hkv, dtype=torch.float64, device=dev)
    mass_k = torch.zeros(w.Hkv, dtype=torch.float64, device=dev)

    def sums(s, o, dq):
        for g in range(w.Hkv):
            hs = slice(g * w.G, (g + 1) * w.G)
            rhs_v[g] += (x["d_o"][:, hs].double() * o[:, hs].double()).sum()
            rhs_k[g] += (dq[:, hs].double() * x["q"][:, hs].double()).sum()
            mass_v[g] += (x["d_o"][:, hs].double().abs() * o[:, hs].double().abs()).sum()
            mass_k[g] += (dq[:, hs].double().abs() * x["q"][:, hs].double().abs()).sum()

    res, lists = _run_sequence(w, x, sums)
    steps = len(lists)
    touched = [set() for _ in range(w.Hkv)]
    for hsel, hcnt in lists:
        for g in range(w.Hkv):
            touched[g] |= set(hsel[g][:hcnt[g]].tolist())

    # the last call against the oracle
    last = w.with_(name="qwen_sparse_1m_last", N=w.N + (steps - 1) * w.C, extra_phys=0)
    assert last.n == w.n_phys
    osel, ocnt, _ = pu.oracle_select(last, hx)
    hsel, hcnt = lists[-1]
    assert np.array_equal(hcnt, ocnt) and np.array_equal(hsel, osel)
    _check_rows(last, hx, res, osel, ocnt, _sample_rows(last, 64, 4))

    # the pools after the 16 calls
    for g in range(w.Hkv):
        lhs_v = (x["dv_pool"][:, g].double() * x["v_pool"][:, g].double()).sum().item()
        lhs_k = (x["dk_pool"][:, g].double() * x["k_pool"][:, g].double()).sum().item()
        assert abs(lhs_v - rhs_v[g].item()) <= 5e-3 * mass_v[g].item(), (g, lhs_v, rhs_v[g].item())
        assert abs(lhs_k - rhs_k[g].item()) <= 5e-3 * mass_k[g].item(), (g, lhs_k, rhs_k[g].item())
        untouched = np.setdiff1d(np.arange(w.n_phys), hx["page_table"][np.array(sorted(touched[g]))])
        idx = torch.as_tensor(untouched, device=dev)
        assert not x["dk_pool"][idx, g].any() and not x["dv_pool"][idx, g].any()


def test_sequence_accumulated_units():
    """Sec. 3 Eq. 3 at the benchmark's size: the gradient of a page is the sum of what the later chunks'
    backward passes add to it.  After the 16 calls, pages of one KV head are compared element by element with
    the oracle run over the same 16 calls (its own selection, forward statistics and dK / dV per call, added
    up in fp32): pages retrieved by every call, a page that is local in the first call and past afterwards, and
    the last call's last local page."""
    w = WORKLOADS["qwen_sparse_1m"]
    x = make_inputs(w, "cuda")
    hx = pu.host_inputs(x)
    res, lists = _run_sequence(w, x)
    steps = len(lists)
    g = 2
    in_all = set(lists[0][0][g][:w.top_k].tolist())
    for hsel, hcnt in lists[1:]:
        in_all &= set(hsel[g][:w.top_k].tolist())
    in_all = sorted(in_all)
    assert len(in_all) >= 3, "the seeded inputs are expected to retrieve some pages in every call"
    pages = [in_all[0], in_all[len(in_all) // 2], in_all[-1], w.n_past, w.n_past + w.m - 1, w.n_phys - 1]
    dk = np.zeros(hx["k_pool"].shape, dtype=np.float32)
    dv = np.zeros(hx["k_pool"].shape, dtype=np.float32)
    n_added = 0
    for s in range(steps):
        ws_ = w.with_(name=f"qwen_sparse_1m_call{s}", N=w.N + s * w.C, extra_phys=w.extra_phys - s * w.m)
        osel, ocnt, _ = pu.oracle_select(ws_, hx)
        assert np.array_equal(lists[s][1], ocnt) and np.array_equal(lists[s][0], osel), f"lists of call {s} differ"
        listed = set(osel[g][:ocnt[g]].tolist())
        mine = [l for l in pages if l in listed]
        n_added += len(mine)
        if mine:
            _oracle_units(ws_, hx, osel, ocnt, g, mine, dk, dv)
    assert n_added >= 3 * steps + 3
    _compare_units(hx, res, g, pages, dk, dv)
