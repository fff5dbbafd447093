"""Python binding of the C-ABI library (include/oomb.h): argument marshalling
only.  Torch supplies device memory and the stream; every step of the path runs
in the library's HIP kernels.  Function names mirror the C entry points."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liboomb.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_LAUNCH, ERR_OUT_OF_PAGES, ERR_SCRATCH_LIMIT = range(7)
NOALLOC_SCRATCH_BYTES = 4 << 20
F32, BF16 = 0, 1
OP_SCORE_TOPK, OP_ATTN_FWD, OP_ATTN_BWD, OP_VOTE_TOPK, OP_ATTN_FWD_QP, OP_ATTN_BWD_QP, \
    OP_CHECK_INPUTS = range(7)

EXPORTS = ["oomb_workspace_bytes", "oomb_page_score_topk", "oomb_paged_attn_fwd",
           "oomb_paged_attn_bwd", "oomb_status_string", "oomb_version", "oomb_profile_enable",
           "oomb_profile_reset", "oomb_profile_count", "oomb_profile_read", "oomb_calibrate",
           "oomb_kv_append", "oomb_page_means", "oomb_page_score_topk_cached", "oomb_local_page_list",
           "oomb_page_pool_reset", "oomb_page_pool_alloc", "oomb_page_pool_release",
           "oomb_paged_attn_fwd_qp", "oomb_paged_attn_bwd_qp", "oomb_page_vote_topk",
           "oomb_offload_plan", "oomb_offload_fetch", "oomb_offload_writeback", "oomb_check_inputs",
           "oomb_page_score_topk_noalloc"]


class AttnDesc(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("page_size", ctypes.c_int32),
                ("chunk_len", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("grad_dtype", ctypes.c_int32), ("sm_scale", ctypes.c_float),
                ("ctx_len", ctypes.c_int64),
                ("pool_page_stride", ctypes.c_int64), ("pool_head_stride", ctypes.c_int64),
                ("pool_tok_stride", ctypes.c_int64),
                ("q_tok_stride", ctypes.c_int64), ("q_head_stride", ctypes.c_int64),
                ("num_phys_pages", ctypes.c_int64)]


class OombError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def lib():
    """The loaded C-ABI library.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2602_02108_amd.build "
                               "or __graft_entry__.build())")
        l = ctypes.CDLL(LIB_PATH)
        vp, i32, u64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        dp = ctypes.POINTER(AttnDesc)
        l.oomb_workspace_bytes.restype = u64
        l.oomb_workspace_bytes.argtypes = [dp, i32, i32]
        l.oomb_page_score_topk.restype = i32
        l.oomb_page_score_topk.argtypes = [dp, vp, vp, vp, i32, vp, vp, vp, vp, u64, vp]
        l.oomb_page_score_topk_noalloc.restype = i32
        l.oomb_page_score_topk_noalloc.argtypes = [dp, vp, vp, vp, i32, vp, vp, vp, vp]
        l.oomb_paged_attn_fwd.restype = i32
        l.oomb_paged_attn_fwd.argtypes = [dp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, u64, vp]
        l.oomb_paged_attn_bwd.restype = i32
        l.oomb_paged_attn_bwd.argtypes = [dp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, u64, vp]
        l.oomb_paged_attn_fwd_qp.restype = i32
        l.oomb_paged_attn_fwd_qp.argtypes = l.oomb_paged_attn_fwd.argtypes
        l.oomb_paged_attn_bwd_qp.restype = i32
        l.oomb_paged_attn_bwd_qp.argtypes = l.oomb_paged_attn_bwd.argtypes
        l.oomb_page_vote_topk.restype = i32
        l.oomb_page_vote_topk.argtypes = [dp, vp, vp, i32, vp, vp, vp, vp, u64, vp]
        l.oomb_offload_plan.restype = i32
        l.oomb_offload_plan.argtypes = [dp, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp]
        l.oomb_offload_fetch.restype = i32
        l.oomb_offload_fetch.argtypes = [dp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp]
        l.oomb_offload_writeback.restype = i32
        l.oomb_offload_writeback.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp]
        l.oomb_check_inputs.restype = i32
        l.oomb_check_inputs.argtypes = [dp, vp, vp, vp, i32, i32, vp, vp, u64, vp]
        l.oomb_status_string.restype = ctypes.c_char_p
        l.oomb_status_string.argtypes = [i32]
        l.oomb_version.restype = i32
        l.oomb_profile_enable.restype = None
        l.oomb_profile_enable.argtypes = [i32]
        l.oomb_profile_reset.restype = None
        l.oomb_profile_count.restype = i32
        l.oomb_profile_read.restype = i32
        l.oomb_profile_read.argtypes = [i32, ctypes.c_char_p, i32, ctypes.POINTER(ctypes.c_double),
                                        ctypes.POINTER(ctypes.c_int64)]
        i64, fp = ctypes.c_int64, ctypes.c_void_p
        l.oomb_kv_append.restype = i32
        l.oomb_kv_append.argtypes = [dp, vp, vp, vp, vp, vp, fp, vp]
        l.oomb_page_means.restype = i32
        l.oomb_page_means.argtypes = [dp, vp, vp, i64, i64, fp, vp]
        l.oomb_page_score_topk_cached.restype = i32
        l.oomb_page_score_topk_cached.argtypes = [dp, vp, fp, i32, vp, vp, vp, vp, u64, vp]
        l.oomb_local_page_list.restype = i32
        l.oomb_local_page_list.argtypes = [dp, i32, vp, vp, vp]
        l.oomb_page_pool_reset.restype = i32
        l.oomb_page_pool_reset.argtypes = [i64, vp, ctypes.POINTER(i64)]
        l.oomb_page_pool_alloc.restype = i32
        l.oomb_page_pool_alloc.argtypes = [vp, ctypes.POINTER(i64), i64, vp]
        l.oomb_page_pool_release.restype = i32
        l.oomb_page_pool_release.argtypes = [i64, vp, ctypes.POINTER(i64), vp, i64]
        l.oomb_calibrate.restype = i32
        l.oomb_calibrate.argtypes = [i32, vp, u64, ctypes.POINTER(ctypes.c_double), vp]
        _lib = l
    return _lib


def status_string(status: int) -> str:
    return lib().oomb_status_string(int(status)).decode()


def version() -> int:
    return int(lib().oomb_version())


def _dt(t: torch.dtype) -> int:
    if t == torch.float32:
        return F32
    if t == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t}")


def make_desc(q: torch.Tensor, k_pool: torch.Tensor, ctx_len: int, sm_scale: float,
              grad_dtype: torch.dtype = torch.float32) -> AttnDesc:
    """Descriptor from a query chunk [C][Hq][D] and a K pool [n_phys][Hkv][P][D]."""
    C, Hq, D = q.shape
    n_phys, Hkv, P, D2 = k_pool.shape
    assert D == D2 and q.stride(2) == 1 and k_pool.stride(3) == 1
    return AttnDesc(Hq, Hkv, D, P, C, _dt(q.dtype), _dt(grad_dtype), float(sm_scale), int(ctx_len),
                    k_pool.stride(0), k_pool.stride(1), k_pool.stride(2), q.stride(0), q.stride(1), n_phys)


def _like(where: str, name: str, t: Optional[torch.Tensor], ref: torch.Tensor, dtype=None) -> None:
    """The descriptor carries ONE stride set for Q / O / dO / dQ and one for the K / V / dK / dV pools: every tensor of
    a family must have the shape and strides of the tensor the descriptor was made from (and the expected dtype)."""
    if t is None:
        return
    want = ref.dtype if dtype is None else dtype
    if tuple(t.shape) != tuple(ref.shape) or tuple(t.stride()) != tuple(ref.stride()) or t.dtype != want:
        raise OombError(ERR_INVALID_ARG, f"{where}: {name} must have shape {tuple(ref.shape)}, strides {tuple(ref.stride())} "
                                         f"and dtype {want} (got {tuple(t.shape)}, {tuple(t.stride())}, {t.dtype})")


def _check_family(where: str, desc: "AttnDesc", q, k_pool, rows=(), pools=(), grad_pools=(), lse=None) -> None:
    if lse is not None and (lse.dtype != torch.float32 or tuple(lse.shape) != (desc.n_q_heads, desc.chunk_len) or
                            not lse.is_contiguous()):
        raise OombError(ERR_INVALID_ARG, f"{where}: lse must be a contiguous float32 [Hq][C] tensor")
    if (q.stride(0), q.stride(1)) != (desc.q_tok_stride, desc.q_head_stride) or _dt(q.dtype) != desc.dtype:
        raise OombError(ERR_INVALID_ARG, f"{where}: q does not match the descriptor's strides / dtype")
    if tuple(k_pool.stride()[:3]) != (desc.pool_page_stride, desc.pool_head_stride, desc.pool_tok_stride):
        raise OombError(ERR_INVALID_ARG, f"{where}: k_pool does not match the descriptor's strides")
    for name, t in rows:
        _like(where, name, t, q)
    for name, t in pools:
        _like(where, name, t, k_pool)
    gdt = torch.bfloat16 if desc.grad_dtype == BF16 else torch.float32
    for name, t in grad_pools:
        _like(where, name, t, k_pool, gdt)


def _p(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(t: torch.Tensor):
    return ctypes.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def workspace_bytes(desc: AttnDesc, top_k: int, op: int) -> int:
    return int(lib().oomb_workspace_bytes(ctypes.byref(desc), int(top_k), int(op)))


def _workspace(desc, top_k, op, device, workspace):
    need = workspace_bytes(desc, top_k, op)
    if need == 0 and op != OP_SCORE_TOPK and top_k < 0:
        need = workspace_bytes(desc, -1, op)
    if need == 0:
        raise OombError(ERR_INVALID_ARG, "oomb_workspace_bytes")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=device)
    return workspace, workspace.numel() * workspace.element_size()


def page_score_topk(desc: AttnDesc, q, k_pool, page_table, top_k: int, sel_pages=None, sel_count=None,
                    scores_out=None, workspace=None):
    """oomb_page_score_topk.  Returns (sel_pages [Hkv][top_k + m] int32, sel_count [Hkv] int32)."""
    m = desc.chunk_len // desc.page_size
    if sel_pages is None:
        sel_pages = torch.empty((desc.n_kv_heads, top_k + m), dtype=torch.int32, device=q.device)
    if sel_count is None:
        sel_count = torch.empty((desc.n_kv_heads,), dtype=torch.int32, device=q.device)
    workspace, nbytes = _workspace(desc, top_k, OP_SCORE_TOPK, q.device, workspace)
    st = lib().oomb_page_score_topk(ctypes.byref(desc), _p(q), _p(k_pool), _p(page_table), int(top_k),
                                    _p(sel_pages), _p(sel_count), _p(scores_out), _p(workspace), nbytes,
                                    _stream(q))
    if st != OK:
        raise OombError(st, "oomb_page_score_topk")
    return sel_pages, sel_count


def page_score_topk_noalloc(desc: AttnDesc, q, k_pool, page_table, top_k: int, sel_pages, sel_count, scores_out=None):
    """oomb_page_score_topk_noalloc: every buffer is the caller's; nothing is allocated here either."""
    st = lib().oomb_page_score_topk_noalloc(ctypes.byref(desc), _p(q), _p(k_pool), _p(page_table), int(top_k),
                                            _p(sel_pages), _p(sel_count), _p(scores_out), _stream(q))
    if st != OK:
        raise OombError(st, "oomb_page_score_topk_noalloc")
    return sel_pages, sel_count


def paged_attn_fwd(desc: AttnDesc, q, k_pool, v_pool, page_table, sel_pages=None, sel_count=None, o=None,
                   lse=None, workspace=None):
    """oomb_paged_attn_fwd.  Returns (O [C][Hq][D], LSE [Hq][C] float32)."""
    if o is None:
        o = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((desc.n_q_heads, desc.chunk_len), dtype=torch.float32, device=q.device)
    _check_family("oomb_paged_attn_fwd", desc, q, k_pool, rows=[("o", o)], pools=[("v_pool", v_pool)], lse=lse)
    stride = 0 if sel_pages is None else int(sel_pages.stride(0))
    list_k = -1 if sel_pages is None else stride - desc.chunk_len // desc.page_size
    workspace, nbytes = _workspace(desc, list_k, OP_ATTN_FWD, q.device, workspace)
    st = lib().oomb_paged_attn_fwd(ctypes.byref(desc), _p(q), _p(k_pool), _p(v_pool), _p(page_table),
                                   _p(sel_pages), _p(sel_count), stride, _p(o), _p(lse), _p(workspace), nbytes,
                                   _stream(q))
    if st != OK:
        raise OombError(st, "oomb_paged_attn_fwd")
    return o, lse


def paged_attn_bwd(desc: AttnDesc, q, k_pool, v_pool, page_table, o, lse, d_o, dk_pool, dv_pool,
                   sel_pages=None, sel_count=None, d_q=None, workspace=None):
    """oomb_paged_attn_bwd.  Returns dQ; dk_pool / dv_pool are accumulated in place."""
    if d_q is None:
        d_q = torch.empty_like(q)
    _check_family("oomb_paged_attn_bwd", desc, q, k_pool, rows=[("o", o), ("d_o", d_o), ("d_q", d_q)],
                  pools=[("v_pool", v_pool)], grad_pools=[("dk_pool", dk_pool), ("dv_pool", dv_pool)], lse=lse)
    stride = 0 if sel_pages is None else int(sel_pages.stride(0))
    list_k = -1 if sel_pages is None else stride - desc.chunk_len // desc.page_size
    workspace, nbytes = _workspace(desc, list_k, OP_ATTN_BWD, q.device, workspace)
    st = lib().oomb_paged_attn_bwd(ctypes.byref(desc), _p(q), _p(k_pool), _p(v_pool), _p(page_table),
                                   _p(sel_pages), _p(sel_count), stride, _p(o), _p(lse), _p(d_o), _p(d_q),
                                   _p(dk_pool), _p(dv_pool), _p(workspace), nbytes, _stream(q))
    if st != OK:
        raise OombError(st, "oomb_paged_attn_bwd")
    return d_q


def page_vote_topk(desc: AttnDesc, q, kbar_cache, top_k: int, sel_pages=None, sel_count=None, votes_out=None,
                   workspace=None):
    """oomb_page_vote_topk.  Returns (sel_pages [Hkv][m][top_k + m] int32, sel_count [Hkv][m] int32)."""
    m = desc.chunk_len // desc.page_size
    if sel_pages is None:
        sel_pages = torch.empty((desc.n_kv_heads, m, top_k + m), dtype=torch.int32, device=q.device)
    if sel_count is None:
        sel_count = torch.empty((desc.n_kv_heads, m), dtype=torch.int32, device=q.device)
    workspace, nbytes = _workspace(desc, top_k, OP_VOTE_TOPK, q.device, workspace)
    st = lib().oomb_page_vote_topk(ctypes.byref(desc), _p(q), _p(kbar_cache), top_k, _p(sel_pages), _p(sel_count),
                                   _p(votes_out), _p(workspace), nbytes, _stream(q))
    if st != OK:
        raise OombError(st, "oomb_page_vote_topk")
    return sel_pages, sel_count


def _stream_of(stream, t):
    return ctypes.c_void_p(stream.cuda_stream) if stream is not None else _stream(t)


def check_inputs(desc: AttnDesc, page_table, sel_pages=None, sel_count=None) -> int:
    """oomb_check_inputs: the violation bits (0 = the documented preconditions hold).  Synchronises."""
    dev = page_table.device
    out = torch.zeros(1, dtype=torch.int32, device=dev)
    ws = torch.empty(max(workspace_bytes(desc, 0, OP_CHECK_INPUTS), 256), dtype=torch.uint8, device=dev)
    stride = lists = 0
    if sel_pages is not None:
        assert sel_pages.dim() in (2, 3) and sel_pages.is_contiguous() and sel_count.is_contiguous()
        stride = int(sel_pages.shape[-1])
        lists = 1 if sel_pages.dim() == 2 else int(sel_pages.shape[1])
    st = lib().oomb_check_inputs(ctypes.byref(desc), _p(page_table), _p(sel_pages), _p(sel_count), stride, lists, _p(out),
                                 _p(ws), ws.numel(), _stream(page_table))
    if st != OK:
        raise OombError(st, "oomb_check_inputs")
    return int(out.item())


class OffloadPlan:
    """Device arrays written by oomb_offload_plan (see include/oomb.h)."""

    def __init__(self, desc, capacity, device):
        n = desc.ctx_len // desc.page_size
        self.capacity = int(capacity)
        self.stage_table = torch.empty(n, dtype=torch.int32, device=device)
        self.slot_pages = torch.empty(self.capacity, dtype=torch.int32, device=device)
        self.head_mask = torch.empty(n, dtype=torch.int32, device=device)   # bit patterns of uint32
        self.n_slots = torch.empty(2, dtype=torch.int32, device=device)   # [slots in use, pages held]

    def overflowed(self) -> bool:
        """True iff the lists held more pages than the staging pools have slots (synchronises)."""
        return int(self.n_slots[1].item()) > self.capacity


def offload_capacity(desc: AttnDesc, sel_pages) -> int:
    """Slots that always suffice for lists of this shape: min(n, Hkv * lists per head * row stride)."""
    n = desc.ctx_len // desc.page_size
    return min(n, sel_pages.numel())


def offload_plan(desc: AttnDesc, sel_pages, sel_count, plan: "OffloadPlan" = None, stream=None) -> "OffloadPlan":
    """oomb_offload_plan for lists [Hkv][stride] or [Hkv][m][stride].  plan.stage_table is the page table to give
    the attention calls that run on the staging pools; plan.capacity must be the staging pools' page count."""
    assert sel_pages.dim() in (2, 3) and sel_pages.is_contiguous() and sel_count.is_contiguous()
    lists_per_head = 1 if sel_pages.dim() == 2 else int(sel_pages.shape[1])
    if plan is None:
        plan = OffloadPlan(desc, offload_capacity(desc, sel_pages), sel_pages.device)
    st = lib().oomb_offload_plan(ctypes.byref(desc), _p(sel_pages), _p(sel_count), int(sel_pages.shape[-1]), lists_per_head,
                                 plan.capacity, _p(plan.stage_table), _p(plan.slot_pages), _p(plan.head_mask), _p(plan.n_slots),
                                 _stream_of(stream, sel_pages))
    if st != OK:
        raise OombError(st, "oomb_offload_plan")
    return plan


def offload_fetch(desc: AttnDesc, host_k_pool, host_v_pool, page_table, plan: "OffloadPlan", stage_k, stage_v,
                  stage_dk=None, stage_dv=None, stream=None) -> None:
    """oomb_offload_fetch: host_*_pool are pinned host tensors (or device tensors) with the pools' layout; the
    staging pools hold stage_k.shape[0] pages."""
    if int(stage_k.shape[0]) != plan.capacity:
        raise OombError(ERR_INVALID_ARG, "oomb_offload_fetch (staging pool size differs from the plan's capacity)")
    _like("oomb_offload_fetch", "host_v_pool", host_v_pool, host_k_pool)
    _like("oomb_offload_fetch", "stage_v", stage_v, stage_k)
    gdt = torch.bfloat16 if desc.grad_dtype == BF16 else torch.float32
    _like("oomb_offload_fetch", "stage_dk", stage_dk, stage_k, gdt)
    _like("oomb_offload_fetch", "stage_dv", stage_dv, stage_k, gdt)
    if tuple(host_k_pool.stride()[1:]) != tuple(stage_k.stride()[1:]) or host_k_pool.dtype != stage_k.dtype or \
            tuple(stage_k.stride()[:3]) != (desc.pool_page_stride, desc.pool_head_stride, desc.pool_tok_stride):
        raise OombError(ERR_INVALID_ARG, "oomb_offload_fetch: host and staging pools must share the descriptor's strides and dtype")
    st = lib().oomb_offload_fetch(ctypes.byref(desc), _p(host_k_pool), _p(host_v_pool), _p(page_table), _p(plan.slot_pages),
                                  _p(plan.head_mask), _p(plan.n_slots), int(stage_k.shape[0]), _p(stage_k), _p(stage_v),
                                  _p(stage_dk), _p(stage_dv), _stream_of(stream, stage_k))
    if st != OK:
        raise OombError(st, "oomb_offload_fetch")


def offload_writeback(desc: AttnDesc, stage_dk, stage_dv, host_dk_pool, host_dv_pool, page_table, plan: "OffloadPlan",
                      stream=None) -> None:
    """oomb_offload_writeback: host pools += the staged gradient tiles of the held (page, KV head) pairs."""
    if int(stage_dk.shape[0]) != plan.capacity:
        raise OombError(ERR_INVALID_ARG, "oomb_offload_writeback (staging pool size differs from the plan's capacity)")
    gdt = torch.bfloat16 if desc.grad_dtype == BF16 else torch.float32
    _like("oomb_offload_writeback", "stage_dv", stage_dv, stage_dk, gdt)
    _like("oomb_offload_writeback", "host_dv_pool", host_dv_pool, host_dk_pool, gdt)
    if tuple(host_dk_pool.stride()[1:]) != tuple(stage_dk.stride()[1:]) or stage_dk.dtype != gdt or \
            tuple(stage_dk.stride()[:3]) != (desc.pool_page_stride, desc.pool_head_stride, desc.pool_tok_stride):
        raise OombError(ERR_INVALID_ARG, "oomb_offload_writeback: host and staging pools must share the descriptor's strides and dtype")
    st = lib().oomb_offload_writeback(ctypes.byref(desc), _p(stage_dk), _p(stage_dv), _p(host_dk_pool), _p(host_dv_pool),
                                      _p(page_table), _p(plan.slot_pages), _p(plan.head_mask), _p(plan.n_slots),
                                      int(stage_dk.shape[0]), _stream_of(stream, stage_dk))
    if st != OK:
        raise OombError(st, "oomb_offload_writeback")


def _qp_lists(desc, sel_pages, sel_count):
    m = desc.chunk_len // desc.page_size
    assert sel_pages.dim() == 3 and sel_pages.shape[:2] == (desc.n_kv_heads, m) and sel_pages.is_contiguous()
    assert sel_count.shape == (desc.n_kv_heads, m) and sel_count.is_contiguous()
    return int(sel_pages.shape[2]), m


def paged_attn_fwd_qp(desc: AttnDesc, q, k_pool, v_pool, page_table, sel_pages, sel_count, o=None, lse=None,
                      workspace=None):
    """oomb_paged_attn_fwd_qp: one list per (KV head, query page), sel_pages [Hkv][m][stride] int32,
    sel_count [Hkv][m].  Returns (O, LSE)."""
    if o is None:
        o = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((desc.n_q_heads, desc.chunk_len), dtype=torch.float32, device=q.device)
    _check_family("oomb_paged_attn_fwd_qp", desc, q, k_pool, rows=[("o", o)], pools=[("v_pool", v_pool)], lse=lse)
    stride, m = _qp_lists(desc, sel_pages, sel_count)
    workspace, nbytes = _workspace(desc, stride - m, OP_ATTN_FWD_QP, q.device, workspace)
    st = lib().oomb_paged_attn_fwd_qp(ctypes.byref(desc), _p(q), _p(k_pool), _p(v_pool), _p(page_table),
                                      _p(sel_pages), _p(sel_count), stride, _p(o), _p(lse), _p(workspace), nbytes,
                                      _stream(q))
    if st != OK:
        raise OombError(st, "oomb_paged_attn_fwd_qp")
    return o, lse


def paged_attn_bwd_qp(desc: AttnDesc, q, k_pool, v_pool, page_table, o, lse, d_o, dk_pool, dv_pool, sel_pages,
                      sel_count, d_q=None, workspace=None):
    """oomb_paged_attn_bwd_qp.  Returns dQ; dk_pool / dv_pool are accumulated in place."""
    if d_q is None:
        d_q = torch.empty_like(q)
    _check_family("oomb_paged_attn_bwd_qp", desc, q, k_pool, rows=[("o", o), ("d_o", d_o), ("d_q", d_q)],
                  pools=[("v_pool", v_pool)], grad_pools=[("dk_pool", dk_pool), ("dv_pool", dv_pool)], lse=lse)
    stride, m = _qp_lists(desc, sel_pages, sel_count)
    workspace, nbytes = _workspace(desc, stride - m, OP_ATTN_BWD_QP, q.device, workspace)
    st = lib().oomb_paged_attn_bwd_qp(ctypes.byref(desc), _p(q), _p(k_pool), _p(v_pool), _p(page_table),
                                      _p(sel_pages), _p(sel_count), stride, _p(o), _p(lse), _p(d_o), _p(d_q),
                                      _p(dk_pool), _p(dv_pool), _p(workspace), nbytes, _stream(q))
    if st != OK:
        raise OombError(st, "oomb_paged_attn_bwd_qp")
    return d_q


def profile_enable(on) -> None:
    """oomb_profile_enable: 1 / True brackets every kernel launch with HIP events on the launch stream,
    2 only the four large kernels, 0 / False none."""
    lib().oomb_profile_enable(int(on))


def profile_reset() -> None:
    lib().oomb_profile_reset()


def profile_read() -> dict:
    """oomb_profile_read for every entry: {kernel name: (total_ms, launches)}."""
    out = {}
    for idx in range(lib().oomb_profile_count()):
        name = ctypes.create_string_buffer(64)
        ms = ctypes.c_double()
        n = ctypes.c_int64()
        st = lib().oomb_profile_read(idx, name, 64, ctypes.byref(ms), ctypes.byref(n))
        if st != OK:
            raise OombError(st, "oomb_profile_read")
        out[name.value.decode()] = (ms.value, n.value)
    return out


def calibrate(which: int, buf) -> float:
    """oomb_calibrate: measured ceiling of the device (0: bf16 MFMA TFLOP/s on constant operands, 2: on random
    operands, 1: copy GB/s, read + write)."""
    out = ctypes.c_double()
    st = lib().oomb_calibrate(int(which), _p(buf), buf.numel() * buf.element_size(), ctypes.byref(out), _stream(buf))
    if st != OK:
        raise OombError(st, "oomb_calibrate")
    return out.value


def kv_append(desc: AttnDesc, k_chunk, v_chunk, page_table, k_pool, v_pool, kbar_cache=None) -> None:
    """oomb_kv_append: the chunk's K / V [C][Hkv][D] into its local pages (+ their means into kbar_cache)."""
    if not (k_chunk.is_contiguous() and v_chunk.is_contiguous()) or k_chunk.shape != v_chunk.shape or \
            k_chunk.dtype != k_pool.dtype or v_chunk.dtype != k_pool.dtype:
        raise OombError(ERR_INVALID_ARG, "oomb_kv_append: k_chunk / v_chunk must be contiguous [C][Hkv][D] of the pools' dtype")
    _like("oomb_kv_append", "v_pool", v_pool, k_pool)
    st = lib().oomb_kv_append(ctypes.byref(desc), _p(k_chunk), _p(v_chunk), _p(page_table), _p(k_pool), _p(v_pool),
                              _p(kbar_cache), _stream(k_pool))
    if st != OK:
        raise OombError(st, "oomb_kv_append")


class PagePool:
    """Free list of the physical pages that the K / V / dK / dV pools share (oomb_page_pool_*): host-side state
    (a stack of page ids and its fill level) held here, every operation done by the library."""

    def __init__(self, num_phys_pages: int):
        self.num_phys_pages = int(num_phys_pages)
        self._stack = (ctypes.c_int32 * max(self.num_phys_pages, 1))()
        self._n_free = ctypes.c_int64(0)
        st = lib().oomb_page_pool_reset(self.num_phys_pages, self._stack, ctypes.byref(self._n_free))
        if st != OK:
            raise OombError(st, "oomb_page_pool_reset")

    @property
    def n_free(self) -> int:
        return int(self._n_free.value)

    def alloc(self, count: int) -> list:
        out = (ctypes.c_int32 * max(int(count), 1))()
        st = lib().oomb_page_pool_alloc(self._stack, ctypes.byref(self._n_free), int(count), out)
        if st != OK:
            raise OombError(st, "oomb_page_pool_alloc")
        return list(out[: int(count)])

    def release(self, pages) -> None:
        pages = [int(x) for x in pages]
        arr = (ctypes.c_int32 * max(len(pages), 1))(*pages)
        st = lib().oomb_page_pool_release(self.num_phys_pages, self._stack, ctypes.byref(self._n_free), arr, len(pages))
        if st != OK:
            raise OombError(st, "oomb_page_pool_release")


def page_means(desc: AttnDesc, k_pool, page_table, first_page: int, n_pages: int, kbar_cache) -> None:
    """oomb_page_means: means of logical pages [first_page, first_page + n_pages) into kbar_cache."""
    st = lib().oomb_page_means(ctypes.byref(desc), _p(k_pool), _p(page_table), int(first_page), int(n_pages),
                               _p(kbar_cache), _stream(k_pool))
    if st != OK:
        raise OombError(st, "oomb_page_means")


def page_score_topk_cached(desc: AttnDesc, q, kbar_cache, top_k: int, sel_pages=None, sel_count=None,
                           scores_out=None, workspace=None):
    """oomb_page_score_topk_cached.  Returns (sel_pages [Hkv][top_k + m] int32, sel_count [Hkv] int32)."""
    m = desc.chunk_len // desc.page_size
    if sel_pages is None:
        sel_pages = torch.empty((desc.n_kv_heads, top_k + m), dtype=torch.int32, device=q.device)
    if sel_count is None:
        sel_count = torch.empty((desc.n_kv_heads,), dtype=torch.int32, device=q.device)
    workspace, nbytes = _workspace(desc, top_k, OP_SCORE_TOPK, q.device, workspace)
    st = lib().oomb_page_score_topk_cached(ctypes.byref(desc), _p(q), _p(kbar_cache), int(top_k), _p(sel_pages),
                                           _p(sel_count), _p(scores_out), _p(workspace), nbytes, _stream(q))
    if st != OK:
        raise OombError(st, "oomb_page_score_topk_cached")
    return sel_pages, sel_count


def local_page_list(desc: AttnDesc, window_pages: int, device, sel_pages=None, sel_count=None):
    """oomb_local_page_list.  Returns (sel_pages [Hkv][window_pages + m] int32, sel_count [Hkv] int32)."""
    m = desc.chunk_len // desc.page_size
    if sel_pages is None:
        sel_pages = torch.empty((desc.n_kv_heads, window_pages + m), dtype=torch.int32, device=device)
    if sel_count is None:
        sel_count = torch.empty((desc.n_kv_heads,), dtype=torch.int32, device=device)
    st = lib().oomb_local_page_list(ctypes.byref(desc), int(window_pages), _p(sel_pages), _p(sel_count),
                                    _stream(sel_pages))
    if st != OK:
        raise OombError(st, "oomb_local_page_list")
    return sel_pages, sel_count
