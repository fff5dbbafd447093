"""GPU parity of the attention with one page list per (KV head, query page) (paper Sec. 4.2: every
query page retrieves its own top-K pages), element by element against the CPU oracle.  The lists
here are seeded random inputs given to both sides; the retrieval that produces such lists is
tested in test_gpu_vote.py."""
import numpy as np
import pytest
import torch

from paper_2602_02108_amd import api
from paper_2602_02108_amd.workloads import WORKLOADS, Workload, make_inputs, torch_dtype

import oracle as orc
import parity_util as pu

pytestmark = pytest.mark.gpu


def rand_qp_lists(w: Workload, k_sel: int, seed: int, popular: int = 0):
    """[Hkv][m][k_sel + m] ascending lists: k_sel distinct past pages (the first `popular` of them drawn
    from a small pool shared by all query pages of the head, so that some pages are held by many
    lists) followed by the local pages n_past .. n_past + tau."""
    rng = np.random.default_rng(seed)
    k_sel = min(k_sel, w.n_past)
    popular = min(popular, k_sel)
    sel = np.full((w.Hkv, w.m, k_sel + w.m), -1, np.int32)
    cnt = np.zeros((w.Hkv, w.m), np.int32)
    for g in range(w.Hkv):
        pool = rng.choice(w.n_past, size=min(w.n_past, popular + 2), replace=False) if popular else np.empty(0, int)
        for tau in range(w.m):
            pop = rng.choice(pool, size=popular, replace=False) if popular else np.empty(0, int)
            rest = np.setdiff1d(np.arange(w.n_past), pop)
            other = rng.choice(rest, size=k_sel - popular, replace=False)
            lst = sorted(set(pop.tolist()) | set(other.tolist())) + list(range(w.n_past, w.n_past + tau + 1))
            sel[g, tau, : len(lst)] = lst
            cnt[g, tau] = len(lst)
    return sel, cnt


def gpu_fwd_bwd_qp(w, x, sel, cnt):
    desc = api.make_desc(x["q"], x["k_pool"], w.N, w.sm_scale, torch_dtype(w.grad_dtype))
    dsel = torch.as_tensor(sel, device="cuda")
    dcnt = torch.as_tensor(cnt, device="cuda")
    o, lse = api.paged_attn_fwd_qp(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], dsel, dcnt)
    dq = api.paged_attn_bwd_qp(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], o, lse, x["d_o"],
                               x["dk_pool"], x["dv_pool"], dsel, dcnt)
    torch.cuda.synchronize()
    return dict(o=o, lse=lse, dq=dq, dk_pool=x["dk_pool"], dv_pool=x["dv_pool"])


def qp_parity(w: Workload, sel, cnt, init_grad=None):
    x = make_inputs(w, "cuda")
    hx = pu.host_inputs(x)
    dk0 = dv0 = None
    if init_grad is not None:
        g = torch.Generator(device="cuda")
        g.manual_seed(w.seed + 77)
        for k in ("dk_pool", "dv_pool"):
            x[k].copy_((torch.randn(x[k].shape, generator=g, device="cuda") * init_grad).to(x[k].dtype))
        dk0 = x["dk_pool"].float().cpu().numpy().copy()
        dv0 = x["dv_pool"].float().cpu().numpy().copy()
    before_k, before_v = x["dk_pool"].clone(), x["dv_pool"].clone()
    res = gpu_fwd_bwd_qp(w, x, sel, cnt)
    ref = orc.attn_fwd_bwd(pu.shape_of(w), hx["q"], hx["k_pool"], hx["v_pool"], hx["page_table"], hx["d_o"], sel, cnt,
                           dk_pool=dk0, dv_pool=dv0, prec="f32")
    rep = {}
    rep["o"] = pu.check("O", pu.f32(res["o"]), ref["o"], w.dtype)
    rep["lse"] = pu.check("LSE", pu.f32(res["lse"]), ref["lse"], "f32" if w.dtype == "f32" else "bf16")
    rep["dq"] = pu.check("dQ", pu.f32(res["dq"]), ref["dq"], w.dtype)
    gd = w.dtype if w.grad_dtype == "f32" else "bf16"
    rep["dk"] = pu.check("dK pool", pu.f32(res["dk_pool"]), ref["dk_pool"], gd)
    rep["dv"] = pu.check("dV pool", pu.f32(res["dv_pool"]), ref["dv_pool"], gd)
    pt = hx["page_table"]
    for g_ in range(w.Hkv):
        pages = np.unique(sel[g_][sel[g_] >= 0])
        untouched = np.setdiff1d(np.arange(w.n_phys), pt[pages])
        if len(untouched):
            idx = torch.as_tensor(untouched, device="cuda")
            assert torch.equal(res["dk_pool"][idx, g_], before_k[idx, g_]), "dK pool: page in no list modified"
            assert torch.equal(res["dv_pool"][idx, g_], before_v[idx, g_]), "dV pool: page in no list modified"
    print(w.name, {k: (f"{v[0]:.2e}", f"{v[1]:.2e}") for k, v in rep.items()}, flush=True)
    return res


# shape-generic kernels: fp32, and bf16 with a page size that has no MFMA kernel
GENERIC = [
    Workload("qp_f32", 4, 2, 64, 16, 96, 16 * 30, None, "f32", "f32", 0.125, extra_phys=3, seed=31),
    Workload("qp_bf16_p64", 8, 2, 128, 64, 256, 64 * 20, None, "bf16", "bf16", 0.088, extra_phys=2, seed=32),
]
# MFMA kernels (P = D = 128).  m = 12 query pages with a shared pool of popular pages: pages held by
# more than 8 lists are cut into several dK/dV work units whose partial sums are added in a second
# pass; G = 7 makes the last row tile of every query page half empty.
MFMA = [
    Workload("qp_mfma_g7", 14, 2, 128, 128, 128 * 12, 128 * 40, None, "bf16", "f32", 0.0884, extra_phys=5, seed=33),
    Workload("qp_mfma_g2_bf16grad", 4, 2, 128, 128, 128 * 5, 128 * 19, None, "bf16", "bf16", 0.0884, extra_phys=1,
             seed=34),
]


@pytest.mark.parametrize("w", GENERIC, ids=lambda w: w.name)
def test_generic_kernels_with_per_query_page_lists(w):
    sel, cnt = rand_qp_lists(w, 5, w.seed + 1, popular=2)
    qp_parity(w, sel, cnt)


@pytest.mark.parametrize("w", MFMA, ids=lambda w: w.name)
def test_mfma_kernels_with_per_query_page_lists(w):
    sel, cnt = rand_qp_lists(w, 6, w.seed + 1, popular=3)
    qp_parity(w, sel, cnt)


def test_mfma_nonzero_pool_and_disjoint_lists():
    w = MFMA[0]
    sel, cnt = rand_qp_lists(w, 2, w.seed + 2, popular=0)
    qp_parity(w, sel, cnt, init_grad=0.5)


def test_only_local_pages_and_no_history():
    w = MFMA[1]
    sel, cnt = rand_qp_lists(w, 0, 1)
    qp_parity(w, sel, cnt)
    w2 = w.with_(name="qp_nohist", N=w.C)
    sel, cnt = rand_qp_lists(w2, 3, 2)
    assert sel.shape[2] == w2.m
    qp_parity(w2, sel, cnt)


def test_equal_lists_reproduce_the_per_head_kernels():
    """Every query page given the per-head list (cut to its visible local pages): same visible sets as
    the one-list-per-head call, so the outputs agree to rounding (the tiles differ)."""
    w = WORKLOADS["mid_sparse_bf16"]
    x = make_inputs(w, "cuda")
    sel1, cnt1, _ = pu.gpu_select(w, x)
    a = pu.gpu_fwd_bwd(w, x, sel1, cnt1)
    a = {k: v.clone() for k, v in a.items()}
    x["dk_pool"].zero_()
    x["dv_pool"].zero_()
    s1 = sel1.cpu().numpy()
    sel = np.full((w.Hkv, w.m, s1.shape[1]), -1, np.int32)
    cnt = np.zeros((w.Hkv, w.m), np.int32)
    for g in range(w.Hkv):
        past = [l for l in s1[g] if 0 <= l < w.n_past]
        for tau in range(w.m):
            lst = past + list(range(w.n_past, w.n_past + tau + 1))
            sel[g, tau, : len(lst)] = lst
            cnt[g, tau] = len(lst)
    b = gpu_fwd_bwd_qp(w, x, sel, cnt)
    for k in ("o", "lse", "dq", "dk_pool", "dv_pool"):
        mx, rel = pu.errors(pu.f32(b[k]), pu.f32(a[k]))
        assert rel < 2e-3, (k, mx, rel)


def test_qp_backward_is_deterministic():
    w = MFMA[0]
    sel, cnt = rand_qp_lists(w, 6, w.seed + 1, popular=3)
    outs = []
    for _ in range(2):
        x = make_inputs(w, "cuda")
        r = gpu_fwd_bwd_qp(w, x, sel, cnt)
        outs.append({k: v.clone() for k, v in r.items()})
    for k in outs[0]:
        assert torch.equal(outs[0][k], outs[1][k]), k


# row-tile geometry: a query page is 4 G blocks of 32 rows -> ceil(4 G / 8) tiles; G = 1 (half a tile per query
# page), 3 (one full + one half tile), 8 (four full tiles), 5 (two full + one half), a single query page (m = 1)
@pytest.mark.parametrize("G,m", [(1, 3), (3, 2), (8, 2), (5, 3), (7, 1)])
def test_mfma_tile_geometry_for_other_group_sizes(G, m):
    w = Workload(f"qp_g{G}_m{m}", 2 * G, 2, 128, 128, 128 * m, 128 * (m + 9), None, "bf16", "f32", 0.0884, extra_phys=1,
                 seed=80 + G)
    sel, cnt = rand_qp_lists(w, 3, w.seed, popular=1)
    qp_parity(w, sel, cnt)


def test_votes_for_other_group_sizes():
    """The vote kernels split a row tile between two query pages when 4 G is not a multiple of 8."""
    from test_gpu_vote import vote_parity
    for G, m in [(1, 4), (3, 3), (5, 2), (8, 2)]:
        w = Workload(f"vote_g{G}_m{m}", 2 * G, 2, 128, 128, 128 * m, 128 * (m + 70), None, "bf16", "f32", 0.0884,
                     boost_frac=0.1, seed=90 + G)
        *_, differ = vote_parity(w, 5)
        assert differ == 0, (G, m, differ)
