"""GPU parity, element by element against the CPU oracle, at sizes the oracle
finishes in seconds (several tiles, ragged tails, edge cases)."""
import numpy as np
import pytest
import torch

from paper_2602_02108_amd import api
from paper_2602_02108_amd.workloads import WORKLOADS, Workload, make_inputs

import parity_util as pu

pytestmark = pytest.mark.gpu


def _show(name, rep):
    print(name, {k: (f"{v[0]:.2e}", f"{v[1]:.2e}") for k, v in rep.items()}, flush=True)


@pytest.mark.parametrize("name", ["tiny_dense", "tiny_sparse"])
def test_tiny_fp32(name):
    rep = pu.full_parity(WORKLOADS[name])
    _show(name, rep)


def test_tiny_fp32_accumulates_into_nonzero_pool():
    rep = pu.full_parity(WORKLOADS["tiny_sparse"], init_grad=1.0)
    _show("tiny_sparse+init", rep)


GENERIC_CASES = [
    # fp32, D=128, three KV heads, top-k larger than what is available on purpose
    Workload("f32_d128", 6, 3, 128, 32, 96, 32 * 21, 50, "f32", "f32", 0.09, extra_phys=2, seed=11),
    # bf16 through the shape-generic kernels (P = 64 has no MFMA kernel), bf16 gradient pool
    Workload("bf16_p64", 8, 2, 128, 64, 192, 64 * 19, 5, "bf16", "bf16", 0.088, extra_phys=3, boost_frac=0.2,
             seed=12),
    # no history at all: the chunk is the whole context
    Workload("f32_nohist", 4, 2, 64, 16, 64, 64, 4, "f32", "f32", 0.125, seed=13),
    # top_k = 0: only the local pages
    Workload("f32_k0", 4, 2, 64, 16, 64, 320, 0, "f32", "f32", 0.125, seed=14),
]


@pytest.mark.parametrize("w", GENERIC_CASES, ids=lambda w: w.name)
def test_generic_kernels(w):
    rep = pu.full_parity(w)
    _show(w.name, rep)


def test_strided_views_are_honoured():
    """Q / O / dO / dQ as slices of a wider buffer and pools with padded rows."""
    w = WORKLOADS["tiny_sparse"]
    x = make_inputs(w, "cuda")
    hx = pu.host_inputs(x)

    def widen(t, pad):
        shape = list(t.shape)
        shape[-2 if t.dim() == 3 else -1] += 0
        big = torch.zeros(t.shape[:-1] + (t.shape[-1] + pad,), dtype=t.dtype, device=t.device)
        big[..., :t.shape[-1]] = t
        return big[..., :t.shape[-1]]

    xs = dict(x)
    for k in ("q", "d_o", "k_pool", "v_pool", "dk_pool", "dv_pool"):
        xs[k] = widen(x[k], 8)
        assert not xs[k].is_contiguous()
    osel, ocnt, _ = pu.oracle_select(w, hx)
    sel, cnt, _ = pu.gpu_select(w, xs)
    torch.cuda.synchronize()
    assert np.array_equal(sel.cpu().numpy(), osel)
    desc = api.make_desc(xs["q"], xs["k_pool"], w.N, w.sm_scale, torch.float32)
    o = widen(torch.empty_like(x["q"]), 8)
    dq = widen(torch.empty_like(x["q"]), 8)
    o, lse = api.paged_attn_fwd(desc, xs["q"], xs["k_pool"], xs["v_pool"], xs["page_table"], sel, cnt, o=o)
    api.paged_attn_bwd(desc, xs["q"], xs["k_pool"], xs["v_pool"], xs["page_table"], o, lse, xs["d_o"],
                       xs["dk_pool"], xs["dv_pool"], sel, cnt, d_q=dq)
    torch.cuda.synchronize()
    ref = pu.oracle_fwd_bwd(w, hx, osel, ocnt)
    pu.check("O", pu.f32(o), ref["o"], "f32")
    pu.check("dQ", pu.f32(dq), ref["dq"], "f32")
    pu.check("dK", pu.f32(xs["dk_pool"]), ref["dk_pool"], "f32")
    pu.check("dV", pu.f32(xs["dv_pool"]), ref["dv_pool"], "f32")


def test_strided_views_are_honoured_by_the_mfma_kernels():
    """The same with bf16 tensors (MFMA kernels: page images of the forward, direct global -> LDS copies of
    pool rows and of Q / dO rows in the backward): Q / O / dO / dQ rows and pool rows padded by 8 elements,
    bf16 gradient pool."""
    w = Workload("bf16_strided", 14, 2, 128, 128, 256, 128 * 11, 3, "bf16", "bf16", 0.0884, extra_phys=2, seed=41)
    x = make_inputs(w, "cuda")
    hx = pu.host_inputs(x)

    def widen(t, pad=8):
        big = torch.zeros(t.shape[:-1] + (t.shape[-1] + pad,), dtype=t.dtype, device=t.device)
        big[..., :t.shape[-1]] = t
        return big[..., :t.shape[-1]]

    xs = dict(x)
    for k in ("q", "d_o", "k_pool", "v_pool", "dk_pool", "dv_pool"):
        xs[k] = widen(x[k])
        assert not xs[k].is_contiguous()
    osel, ocnt, _ = pu.oracle_select(w, hx)
    sel, cnt, _ = pu.gpu_select(w, xs)
    torch.cuda.synchronize()
    assert np.array_equal(sel.cpu().numpy(), osel)
    desc = api.make_desc(xs["q"], xs["k_pool"], w.N, w.sm_scale, torch.bfloat16)
    o = widen(torch.empty_like(x["q"]))
    dq = widen(torch.empty_like(x["q"]))
    o, lse = api.paged_attn_fwd(desc, xs["q"], xs["k_pool"], xs["v_pool"], xs["page_table"], sel, cnt, o=o)
    api.paged_attn_bwd(desc, xs["q"], xs["k_pool"], xs["v_pool"], xs["page_table"], o, lse, xs["d_o"],
                       xs["dk_pool"], xs["dv_pool"], sel, cnt, d_q=dq)
    torch.cuda.synchronize()
    ref = pu.oracle_fwd_bwd(w, hx, osel, ocnt)
    pu.check("O", pu.f32(o), ref["o"], "bf16")
    pu.check("dQ", pu.f32(dq), ref["dq"], "bf16")
    pu.check("dK", pu.f32(xs["dk_pool"]), ref["dk_pool"], "bf16")
    pu.check("dV", pu.f32(xs["dv_pool"]), ref["dv_pool"], "bf16")


def test_mfma_backward_is_deterministic():
    """bf16 path (sliced dK/dV with the fixed-order reduce): two runs give identical bits."""
    w = WORKLOADS["mid_sparse_bf16"]
    outs = []
    for _ in range(2):
        x = make_inputs(w, "cuda")
        sel, cnt, _ = pu.gpu_select(w, x)
        r = pu.gpu_fwd_bwd(w, x, sel, cnt)
        outs.append({k: v.clone() for k, v in r.items()})
    for k in outs[0]:
        assert torch.equal(outs[0][k], outs[1][k]), k


def test_backward_is_deterministic():
    """Page ownership instead of atomics: two runs give identical bits."""
    w = WORKLOADS["tiny_sparse"]
    outs = []
    for _ in range(2):
        x = make_inputs(w, "cuda")
        sel, cnt, _ = pu.gpu_select(w, x)
        r = pu.gpu_fwd_bwd(w, x, sel, cnt)
        outs.append({k: v.clone() for k, v in r.items()})
    for k in outs[0]:
        assert torch.equal(outs[0][k], outs[1][k]), k


@pytest.mark.parametrize("name", ["smoke_bf16", "mid_sparse_bf16", "mid_dense_bf16"])
def test_mfma_bf16(name):
    rep = pu.full_parity(WORKLOADS[name])
    _show(name, rep)


def test_mfma_bf16_nonzero_pool_and_single_local_page():
    # chunk of one page, history of three pages, G = 1
    w = Workload("bf16_g1", 2, 2, 128, 128, 128, 512, 2, "bf16", "f32", 0.0884, seed=31)
    rep = pu.full_parity(w, init_grad=0.5)
    _show(w.name, rep)


# Stage counts of the dK/dV kernel around its ring of four stage buffers (a slice of a page visits
# (C / 32) G / 2 / n_split 64-row stages, fewer on the causal diagonal): slices of 0 / 1 stages, of 1 / 2,
# of 5 (the ring wraps), and two stages per workgroup with the pool updated in place (one slice).
RING_CASES = [
    Workload("bf16_ring_1", 4, 4, 128, 128, 256, 128 * 8, 2, "bf16", "f32", 0.0884, seed=51),
    Workload("bf16_ring_1_2", 6, 2, 128, 128, 128, 128 * 5, None, "bf16", "bf16", 0.0884, seed=52),
    Workload("bf16_ring_5", 2, 1, 128, 128, 640, 128 * 9, 2, "bf16", "f32", 0.0884, seed=53),
    Workload("bf16_ring_in_place", 4, 4, 128, 128, 128, 128 * 512, None, "bf16", "f32", 0.0884, seed=54),
]


@pytest.mark.parametrize("w", RING_CASES, ids=lambda w: w.name)
def test_mfma_bf16_stage_ring_edges(w):
    with pu.kernels_ran(pu.MFMA_KERNELS):
        rep = pu.full_parity(w, init_grad=0.25)
    _show(w.name, rep)
