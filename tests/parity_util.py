"""Shared helpers of the GPU parity tests: run the HIP path through the C-ABI
binding, run the CPU oracle on the same seeded inputs, compare."""
from __future__ import annotations

import contextlib

import numpy as np
import torch

import oracle as orc
from oracle import Shape
from paper_2602_02108_amd import api
from paper_2602_02108_amd.workloads import Workload, make_inputs, to_numpy, torch_dtype

# tolerances (the benchmark spec): bf16 tensors max-abs 2e-2 and rel-L2 5e-3; fp32 runs rel-L2 1e-4
TOL = {"bf16": dict(max_abs=2e-2, rel_l2=5e-3), "f32": dict(max_abs=1e-3, rel_l2=1e-4)}


MFMA_KERNELS = ("attn_fwd_mfma", "bwd_dq_mfma", "bwd_dkv_mfma")


@contextlib.contextmanager
def kernels_ran(names=MFMA_KERNELS, absent=("attn_fwd_generic", "attn_bwd_generic", "delta")):
    """Asserts that the library launched every kernel in `names` (and none in `absent`) inside the block:
    a bf16 test that silently ran the generic fp32 kernels would still pass its tolerances."""
    api.profile_reset()
    api.profile_enable(1)
    try:
        yield
        torch.cuda.synchronize()
        seen = api.profile_read()
    finally:
        api.profile_enable(0)
        api.profile_reset()
    for k in names:
        assert k in seen and seen[k][1] > 0, f"kernel {k} did not run; launched: {sorted(seen)}"
    for k in absent:
        assert k not in seen, f"kernel {k} ran; launched: {sorted(seen)}"


def shape_of(w: Workload) -> Shape:
    return Shape(w.Hq, w.Hkv, w.D, w.P, w.C, w.N, w.sm_scale)


def errors(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    max_abs = float(np.abs(got - want).max()) if got.size else 0.0
    rel = float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30))
    return max_abs, rel


def check(name, got, want, dtype):
    max_abs, rel = errors(got, want)
    tol = TOL[dtype]
    assert np.isfinite(np.asarray(got, dtype=np.float64)).all(), f"{name}: non-finite output"
    assert max_abs <= tol["max_abs"] and rel <= tol["rel_l2"], \
        f"{name}: max_abs {max_abs:.3e} (tol {tol['max_abs']}), rel_l2 {rel:.3e} (tol {tol['rel_l2']})"
    return max_abs, rel


def f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def gpu_select(w: Workload, x: dict, want_scores=True):
    desc = api.make_desc(x["q"], x["k_pool"], w.N, w.sm_scale, torch_dtype(w.grad_dtype))
    scores = torch.empty((w.Hkv, max(w.n_past, 1)), dtype=torch.float32, device=x["q"].device) if want_scores else None
    sel, cnt = api.page_score_topk(desc, x["q"], x["k_pool"], x["page_table"], w.top_k, scores_out=scores)
    return sel, cnt, (scores[:, :w.n_past] if scores is not None else None)


def gpu_fwd_bwd(w: Workload, x: dict, sel=None, cnt=None):
    """One pass of the HIP path.  Accumulates into x['dk_pool'] / x['dv_pool']."""
    desc = api.make_desc(x["q"], x["k_pool"], w.N, w.sm_scale, torch_dtype(w.grad_dtype))
    o, lse = api.paged_attn_fwd(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], sel, cnt)
    dq = api.paged_attn_bwd(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], o, lse, x["d_o"],
                            x["dk_pool"], x["dv_pool"], sel, cnt)
    torch.cuda.synchronize()
    return dict(o=o, lse=lse, dq=dq, dk_pool=x["dk_pool"], dv_pool=x["dv_pool"])


def host_inputs(x: dict) -> dict:
    return {k: to_numpy(v) for k, v in x.items() if isinstance(v, torch.Tensor) and k not in ("dk_pool", "dv_pool")}


def oracle_select(w: Workload, hx: dict):
    return orc.page_score_topk(shape_of(w), hx["q"], hx["k_pool"], hx["page_table"], w.top_k)


def oracle_fwd_bwd(w: Workload, hx: dict, sel=None, cnt=None, dk0=None, dv0=None):
    return orc.attn_fwd_bwd(shape_of(w), hx["q"], hx["k_pool"], hx["v_pool"], hx["page_table"], hx["d_o"],
                            sel, cnt, dk_pool=dk0, dv_pool=dv0, prec="f32")


def full_parity(w: Workload, device="cuda", init_grad=None):
    """Element-by-element comparison of a whole pass (selection included when the
    workload is sparse).  Returns the error table."""
    x = make_inputs(w, device)
    hx = host_inputs(x)
    report = {}
    sel = cnt = osel = ocnt = None
    if w.top_k is not None:
        sel, cnt, scores = gpu_select(w, x)
        torch.cuda.synchronize()
        osel, ocnt, oscores = oracle_select(w, hx)
        # bit-exact scores, counts and page ids
        assert np.array_equal(scores.cpu().numpy().view(np.uint32), oscores.view(np.uint32)), "scores differ"
        assert np.array_equal(cnt.cpu().numpy(), ocnt), "sel_count differs"
        assert np.array_equal(sel.cpu().numpy(), osel), "selected pages differ"
    dk0 = dv0 = None
    if init_grad is not None:
        g = torch.Generator(device=device)
        g.manual_seed(w.seed + 77)
        for k in ("dk_pool", "dv_pool"):
            x[k].copy_((torch.randn(x[k].shape, generator=g, device=device) * init_grad).to(x[k].dtype))
        dk0 = x["dk_pool"].float().cpu().numpy().copy()
        dv0 = x["dv_pool"].float().cpu().numpy().copy()
    before_k = x["dk_pool"].clone()
    before_v = x["dv_pool"].clone()
    res = gpu_fwd_bwd(w, x, sel, cnt)
    ref = oracle_fwd_bwd(w, hx, osel, ocnt, dk0, dv0)
    report["o"] = check("O", f32(res["o"]), ref["o"], w.dtype)
    report["lse"] = check("LSE", f32(res["lse"]), ref["lse"], "f32" if w.dtype == "f32" else "bf16")
    report["dq"] = check("dQ", f32(res["dq"]), ref["dq"], w.dtype)
    gd = w.dtype if w.grad_dtype == "f32" else "bf16"
    report["dk"] = check("dK pool", f32(res["dk_pool"]), ref["dk_pool"], gd)
    report["dv"] = check("dV pool", f32(res["dv_pool"]), ref["dv_pool"], gd)
    # pages outside the lists (and unreferenced physical pages) are bit-identical
    pt = hx["page_table"]
    for g_ in range(w.Hkv):
        pages = np.arange(w.n) if osel is None else osel[g_][:ocnt[g_]]
        untouched = np.setdiff1d(np.arange(w.n_phys), pt[pages])
        if len(untouched):
            idx = torch.as_tensor(untouched, device=device)
            assert torch.equal(res["dk_pool"][idx, g_], before_k[idx, g_]), "dK pool: unselected page modified"
            assert torch.equal(res["dv_pool"][idx, g_], before_v[idx, g_]), "dV pool: unselected page modified"
    return report
