"""Host-side checks of the C-ABI boundary that need no GPU: the library loads,
exports every symbol the header declares, and rejects bad arguments before any
launch."""
import ctypes
import os
import re

import pytest

from paper_2602_02108_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _good_desc(**kw):
    d = api.AttnDesc(28, 4, 128, 128, 4096, api.BF16, api.F32, 1.0, 65536, 4 * 128 * 128, 128 * 128, 128,
                     28 * 128, 128, 512)
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "oomb.h")).read()
    bench_header = open(os.path.join(ROOT, "include", "oomb_bench.h")).read()
    # the product header holds no entry point that waits for the device: those live in oomb_bench.h
    assert not re.search(r"\boomb_(profile|calibrate)", header)
    declared = set(re.findall(r"\b(oomb_[a-z_]+)\s*\(", header + bench_header))
    assert declared == set(api.EXPORTS)
    l = api.lib()
    for name in declared:
        assert hasattr(l, name), name
    assert api.version() >= 100
    assert api.status_string(api.OK) == "ok"
    assert "unsupported" in api.status_string(api.ERR_UNSUPPORTED)


def test_descriptor_struct_matches_header_layout():
    # int32 x7, float, then int64 x7: no padding surprises
    assert ctypes.sizeof(api.AttnDesc) == 8 * 4 + 7 * 8
    assert api.AttnDesc.ctx_len.offset == 32


def test_workspace_sizes():
    d = _good_desc()
    assert api.workspace_bytes(d, 64, api.OP_SCORE_TOPK) >= (28 * 32 * 128 + 4 * 128 + 4 * 480) * 4
    assert api.workspace_bytes(d, -1, api.OP_ATTN_BWD) >= 28 * 4096 * 4
    # a short sparse list is split over more workgroups and needs room for their partial sums
    assert api.workspace_bytes(d, 64, api.OP_ATTN_BWD) > api.workspace_bytes(d, -1, api.OP_ATTN_BWD)
    assert api.workspace_bytes(d, 0, api.OP_ATTN_FWD) > 0
    # forward: one K and one V image of 32 KiB per (KV head, list entry); a dense call lists all n pages
    m, n = 4096 // 128, 65536 // 128
    assert api.workspace_bytes(d, 64, api.OP_ATTN_FWD) >= 4 * (64 + m) * 2 * 32768
    assert api.workspace_bytes(d, -1, api.OP_ATTN_FWD) >= 4 * n * 2 * 32768
    assert api.workspace_bytes(d, 64, api.OP_ATTN_FWD) < api.workspace_bytes(d, -1, api.OP_ATTN_FWD)
    assert api.workspace_bytes(d, 0, 99) == 0
    assert api.workspace_bytes(_good_desc(chunk_len=4000), 0, api.OP_ATTN_FWD) == 0


@pytest.mark.parametrize("kw,want", [
    (dict(n_kv_heads=5), api.ERR_INVALID_ARG),          # Hq % Hkv != 0
    (dict(chunk_len=4100), api.ERR_INVALID_ARG),        # C % P != 0
    (dict(ctx_len=65000), api.ERR_INVALID_ARG),         # N % P != 0
    (dict(ctx_len=2048), api.ERR_INVALID_ARG),          # N < C
    (dict(sm_scale=0.0), api.ERR_INVALID_ARG),
    (dict(dtype=7), api.ERR_INVALID_ARG),
    (dict(pool_tok_stride=100), api.ERR_INVALID_ARG),   # row shorter than D
    (dict(q_head_stride=132), api.ERR_INVALID_ARG),     # breaks 16-byte row alignment
    (dict(num_phys_pages=100), api.ERR_INVALID_ARG),    # fewer physical pages than logical
    (dict(head_dim=96, pool_tok_stride=96, q_head_stride=96), api.ERR_UNSUPPORTED),
    (dict(page_size=8, num_phys_pages=8192), api.ERR_UNSUPPORTED),
])
def test_bad_descriptors_are_rejected_before_launch(kw, want):
    d = _good_desc(**kw)
    fake = ctypes.c_void_p(0x1000)   # never dereferenced: validation fails first
    l = api.lib()
    st = l.oomb_paged_attn_fwd(ctypes.byref(d), fake, fake, fake, fake, None, None, 0, fake, fake, fake, 1 << 30, None)
    assert st == want
    st = l.oomb_paged_attn_bwd(ctypes.byref(d), fake, fake, fake, fake, None, None, 0, fake, fake, fake, fake, fake,
                               fake, fake, 1 << 30, None)
    assert st == want
    st = l.oomb_page_score_topk(ctypes.byref(d), fake, fake, fake, 4, fake, fake, None, fake, 1 << 30, None)
    assert st == want


def test_null_pointers_and_workspace_are_rejected():
    d = _good_desc()
    l = api.lib()
    fake = ctypes.c_void_p(0x1000)
    assert l.oomb_paged_attn_fwd(ctypes.byref(d), None, fake, fake, fake, None, None, 0, fake, fake, fake, 256,
                                 None) == api.ERR_INVALID_ARG
    assert l.oomb_paged_attn_fwd(None, fake, fake, fake, fake, None, None, 0, fake, fake, fake, 256,
                                 None) == api.ERR_INVALID_ARG
    # misaligned tensor pointer
    assert l.oomb_paged_attn_fwd(ctypes.byref(d), ctypes.c_void_p(0x1004), fake, fake, fake, None, None, 0, fake,
                                 fake, fake, 256, None) == api.ERR_INVALID_ARG
    # selection list without counts, or a row stride that cannot hold the local pages
    assert l.oomb_paged_attn_fwd(ctypes.byref(d), fake, fake, fake, fake, fake, None, 96, fake, fake, fake, 256,
                                 None) == api.ERR_INVALID_ARG
    assert l.oomb_paged_attn_fwd(ctypes.byref(d), fake, fake, fake, fake, fake, fake, 8, fake, fake, fake, 256,
                                 None) == api.ERR_INVALID_ARG
    # forward: workspace missing or too small for the page images
    assert l.oomb_paged_attn_fwd(ctypes.byref(d), fake, fake, fake, fake, None, None, 0, fake, fake, None, 0,
                                 None) == api.ERR_WORKSPACE
    assert l.oomb_paged_attn_fwd(ctypes.byref(d), fake, fake, fake, fake, None, None, 0, fake, fake, fake, 256,
                                 None) == api.ERR_WORKSPACE
    # backward / scoring: workspace missing or too small
    assert l.oomb_paged_attn_bwd(ctypes.byref(d), fake, fake, fake, fake, None, None, 0, fake, fake, fake, fake,
                                 fake, fake, None, 0, None) == api.ERR_WORKSPACE
    assert l.oomb_paged_attn_bwd(ctypes.byref(d), fake, fake, fake, fake, None, None, 0, fake, fake, fake, fake,
                                 fake, fake, fake, 1024, None) == api.ERR_WORKSPACE
    assert l.oomb_page_score_topk(ctypes.byref(d), fake, fake, fake, 4, fake, fake, None, fake, 16,
                                  None) == api.ERR_WORKSPACE
    assert l.oomb_page_score_topk(ctypes.byref(d), fake, fake, fake, -1, fake, fake, None, fake, 1 << 30,
                                  None) == api.ERR_INVALID_ARG
    # more than 2^20 past pages is refused by the selection kernel
    big = _good_desc(ctx_len=(1 << 21) * 128, num_phys_pages=1 << 21)
    assert l.oomb_page_score_topk(ctypes.byref(big), fake, fake, fake, 4, fake, fake, None, fake, 1 << 40,
                                  None) == api.ERR_UNSUPPORTED


def test_calibrate_rejects_bad_arguments_before_launch():
    l = api.lib()
    out = ctypes.c_double()
    fake = ctypes.c_void_p(0x1000)
    assert l.oomb_calibrate(0, None, 1 << 20, ctypes.byref(out), None) == api.ERR_INVALID_ARG
    assert l.oomb_calibrate(0, fake, 1 << 20, None, None) == api.ERR_INVALID_ARG
    assert l.oomb_calibrate(1, ctypes.c_void_p(0x1004), 1 << 20, ctypes.byref(out), None) == api.ERR_INVALID_ARG
    assert l.oomb_calibrate(1, fake, 16, ctypes.byref(out), None) == api.ERR_INVALID_ARG


def test_per_query_page_entry_points_validate_before_launch():
    d = _good_desc()
    l = api.lib()
    fake = ctypes.c_void_p(0x1000)
    m = 4096 // 128
    need_f = api.workspace_bytes(d, 64, api.OP_ATTN_FWD_QP)
    need_b = api.workspace_bytes(d, 64, api.OP_ATTN_BWD_QP)
    # worst case: the m lists of a KV head share no page -> images of min(n, m * (64 + m)) pages per head
    n = 65536 // 128
    assert need_f >= 4 * min(n, m * (64 + m)) * 2 * 32768
    assert need_b > need_f
    assert api.workspace_bytes(d, -1, api.OP_ATTN_FWD_QP) == 0
    # lists are mandatory, with counts and a row stride that holds the local pages
    assert l.oomb_paged_attn_fwd_qp(ctypes.byref(d), fake, fake, fake, fake, None, None, 96, fake, fake, fake,
                                    need_f, None) == api.ERR_INVALID_ARG
    assert l.oomb_paged_attn_fwd_qp(ctypes.byref(d), fake, fake, fake, fake, fake, fake, 8, fake, fake, fake,
                                    need_f, None) == api.ERR_INVALID_ARG
    assert l.oomb_paged_attn_fwd_qp(ctypes.byref(d), fake, fake, fake, fake, fake, fake, 64 + m, fake, fake, fake,
                                    need_f - 1, None) == api.ERR_WORKSPACE
    assert l.oomb_paged_attn_bwd_qp(ctypes.byref(d), fake, fake, fake, fake, fake, fake, 64 + m, fake, fake, fake,
                                    fake, fake, fake, None, 0, None) == api.ERR_WORKSPACE
    assert l.oomb_paged_attn_bwd_qp(ctypes.byref(d), fake, fake, fake, fake, fake, fake, 64 + m, fake, fake, None,
                                    fake, fake, fake, fake, need_b, None) == api.ERR_INVALID_ARG


def test_offload_entry_points_validate_before_launch():
    d = _good_desc()
    l = api.lib()
    fake = ctypes.c_void_p(0x1000)
    m = 4096 // 128
    # plan: row stride that cannot hold the local pages; missing counts; lists per head neither 1 nor m
    assert l.oomb_offload_plan(ctypes.byref(d), fake, fake, 8, 1, 640, fake, fake, fake, fake, None) == api.ERR_INVALID_ARG
    assert l.oomb_offload_plan(ctypes.byref(d), fake, None, 64 + m, 1, 640, fake, fake, fake, fake, None) == api.ERR_INVALID_ARG
    assert l.oomb_offload_plan(ctypes.byref(d), fake, fake, 64 + m, 3, 640, fake, fake, fake, fake, None) == api.ERR_INVALID_ARG
    # staging pools without a page
    assert l.oomb_offload_plan(ctypes.byref(d), fake, fake, 64 + m, 1, 0, fake, fake, fake, fake, None) == api.ERR_INVALID_ARG
    # gradient staging pools come in pairs
    assert l.oomb_offload_fetch(ctypes.byref(d), fake, fake, fake, fake, fake, fake, 640, fake, fake, fake, None,
                                None) == api.ERR_INVALID_ARG
    # a host pool the device cannot address (here: not memory at all) is refused before any launch
    assert l.oomb_offload_fetch(ctypes.byref(d), fake, fake, fake, fake, fake, fake, 640, fake, fake, None, None,
                                None) == api.ERR_INVALID_ARG
    assert l.oomb_offload_fetch(ctypes.byref(d), fake, fake, fake, fake, fake, fake, 0, fake, fake, None, None,
                                None) == api.ERR_INVALID_ARG
    assert l.oomb_offload_writeback(ctypes.byref(d), fake, fake, fake, fake, fake, fake, fake, fake, 640,
                                    None) == api.ERR_INVALID_ARG
    assert l.oomb_offload_writeback(ctypes.byref(d), fake, fake, None, fake, fake, fake, fake, fake, 640,
                                    None) == api.ERR_INVALID_ARG


def test_check_inputs_validates_before_launch():
    d = _good_desc()
    l = api.lib()
    fake = ctypes.c_void_p(0x1000)
    need = api.workspace_bytes(d, 0, api.OP_CHECK_INPUTS)
    assert need >= 512 * 4
    assert l.oomb_check_inputs(ctypes.byref(d), None, None, None, 0, 0, fake, fake, need, None) == api.ERR_INVALID_ARG
    assert l.oomb_check_inputs(ctypes.byref(d), fake, fake, None, 96, 1, fake, fake, need, None) == api.ERR_INVALID_ARG
    assert l.oomb_check_inputs(ctypes.byref(d), fake, fake, fake, 96, 5, fake, fake, need, None) == api.ERR_INVALID_ARG
    assert l.oomb_check_inputs(ctypes.byref(d), fake, None, None, 0, 0, fake, fake, need - 1, None) == api.ERR_WORKSPACE


def test_noalloc_scoring_refuses_shapes_beyond_its_scratch():
    # Hq * m * D floats of query-page sums alone: 64 * 512 * 128 * 4 B = 16 MiB > the 4 MiB built-in array
    d = _good_desc(n_q_heads=64, chunk_len=65536, ctx_len=131072, num_phys_pages=1024, q_tok_stride=64 * 128)
    assert api.workspace_bytes(d, 8, api.OP_SCORE_TOPK) > api.NOALLOC_SCRATCH_BYTES
    fake = ctypes.c_void_p(0x1000)   # never dereferenced: the size check comes before any launch
    st = api.lib().oomb_page_score_topk_noalloc(ctypes.byref(d), fake, fake, fake, 8, fake, fake, None, None)
    assert st == api.ERR_SCRATCH_LIMIT
    assert "scratch" in api.status_string(api.ERR_SCRATCH_LIMIT)
    # bad arguments are still reported first
    st = api.lib().oomb_page_score_topk_noalloc(ctypes.byref(_good_desc()), fake, None, fake, 8, fake, fake, None, None)
    assert st == api.ERR_INVALID_ARG


def test_binding_refuses_tensors_that_do_not_share_the_descriptor_layout():
    """One stride set per tensor family: a dO that comes out of autograd with other strides, a gradient pool of
    another dtype or a differently padded V pool would be addressed wrongly, so the binding refuses them."""
    import torch
    C, Hq, Hkv, D, P, n = 32, 2, 1, 64, 16, 4
    q = torch.zeros(C, Hq, D)
    k = torch.zeros(n, Hkv, P, D)
    desc = api.make_desc(q, k, n * P, 0.125)
    pt = torch.arange(n, dtype=torch.int32)
    lse = torch.zeros(Hq, C)
    strided = torch.zeros(C, Hq, 2 * D)[:, :, :D]            # same shape, other strides
    with pytest.raises(api.OombError, match="d_o"):
        api.paged_attn_bwd(desc, q, k, k, pt, q, lse, strided, k.clone(), k.clone())
    with pytest.raises(api.OombError, match="dk_pool"):
        api.paged_attn_bwd(desc, q, k, k, pt, q, lse, q, k.to(torch.bfloat16), k.clone())
    with pytest.raises(api.OombError, match="v_pool"):
        api.paged_attn_fwd(desc, q, k, torch.zeros(n, Hkv, P + 1, D)[:, :, :P], pt)
    with pytest.raises(api.OombError, match="lse"):
        api.paged_attn_bwd(desc, q, k, k, pt, q, lse.double(), q, k.clone(), k.clone())
    with pytest.raises(api.OombError, match="descriptor"):
        api.paged_attn_fwd(desc, strided, k, k, pt)
