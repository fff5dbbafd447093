"""CPU oracle (test infrastructure) for OOMB's paged sparse attention hot path.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It wraps ``oomb_oracle.c`` (plain C, compiled twice: float and
double arithmetic) through ctypes and exposes numpy-in / numpy-out functions.
It shares nothing with the HIP path.

Paper passages followed: Sec. 3 Eq. 2-3 (chunk attends to the growing KV cache,
KV gradients accumulate), Sec. 4.1 (paged K/V and gradient pools), Sec. 4.2
(page-mean keys, query-aggregated page scores, top-K pages, indices reused by
the backward pass).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_BUILD = os.path.join(_HERE, "_build")
_SRC = os.path.join(_HERE, "oomb_oracle.c")


def build(force: bool = False) -> None:
    """Compile the oracle for float and double arithmetic (gcc, OpenMP)."""
    os.makedirs(_BUILD, exist_ok=True)
    for name, real in (("f32", "float"), ("f64", "double")):
        out = os.path.join(_BUILD, f"liboomb_oracle_{name}.so")
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O2", "-ftree-vectorize", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               f"-DREAL={real}", "-o", out, _SRC, "-lm"]
        subprocess.check_call(cmd)


class _Desc(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("page_size", ctypes.c_int32),
                ("chunk_len", ctypes.c_int32), ("in_is_bf16", ctypes.c_int32),
                ("ctx_len", ctypes.c_int64), ("sm_scale", ctypes.c_double),
                ("lists_per_query_page", ctypes.c_int32)]


@dataclass
class Shape:
    """Problem shape in the paper's notation (Sec. 4.2): C = m*P query tokens,
    N = n*P tokens reachable through the page table (the chunk included)."""
    Hq: int
    Hkv: int
    D: int
    P: int
    C: int
    N: int
    sm_scale: float

    @property
    def n(self) -> int:
        return self.N // self.P

    @property
    def m(self) -> int:
        return self.C // self.P

    @property
    def n_past(self) -> int:
        return self.n - self.m

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv


_libs: dict = {}


def _lib(prec: str):
    if prec not in _libs:
        build()
        lib = ctypes.CDLL(os.path.join(_BUILD, f"liboomb_oracle_{prec}.so"))
        lib.oomb_oracle_row_probs.restype = ctypes.c_int64
        lib.oomb_oracle_real_bytes.restype = ctypes.c_int
        assert lib.oomb_oracle_real_bytes() == (4 if prec == "f32" else 8)
        _libs[prec] = lib
    return _libs[prec]


def num_threads() -> int:
    """Threads the OpenMP loops of the attention functions use."""
    return int(_lib("f32").oomb_oracle_num_threads())


def _real(prec: str):
    return np.float32 if prec == "f32" else np.float64


def _ptr(a):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _inputs(prec, *arrays):
    """Inputs are either all uint16 (bf16 bit patterns) or floating arrays that
    are converted to the oracle's arithmetic type."""
    bf = [a.dtype == np.uint16 for a in arrays]
    if all(bf):
        return 1, [np.ascontiguousarray(a) for a in arrays]
    if any(bf):
        raise ValueError("mix of bf16 and floating inputs")
    return 0, [np.ascontiguousarray(a, dtype=_real(prec)) for a in arrays]


def _desc(sh: Shape, is_bf16: int, per_query_page: int = 0) -> _Desc:
    assert sh.Hq % sh.Hkv == 0 and sh.C % sh.P == 0 and sh.N % sh.P == 0 and sh.N >= sh.C
    return _Desc(sh.Hq, sh.Hkv, sh.D, sh.P, sh.C, is_bf16, sh.N, float(sh.sm_scale), per_query_page)


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _sel_args(sel, sel_count):
    """-> (sel, sel_count, row stride, lists per query page?).  A 2-d sel [Hkv][stride] is one list per
    KV head; a 3-d sel [Hkv][m][stride] (sel_count [Hkv][m]) is one list per KV head and query page."""
    if sel is None:
        return None, None, 0, 0
    sel = _i32(sel)
    cnt = _i32(sel_count)
    assert sel.ndim in (2, 3) and cnt.shape == sel.shape[:-1]
    return sel, cnt, int(sel.shape[-1]), int(sel.ndim == 3)


def page_score_topk(sh: Shape, q, k_pool, page_table, top_k: int):
    """Returns (sel [Hkv][top_k + m] int32, padded with -1; sel_count [Hkv];
    scores [Hkv][n_past] float32).  fp32 arithmetic in a fixed order."""
    bf, (q, k_pool) = _inputs("f32", q, k_pool)
    pt = _i32(page_table)
    assert pt.shape[0] >= sh.n
    sel = np.full((sh.Hkv, top_k + sh.m), -1, dtype=np.int32)
    cnt = np.zeros(sh.Hkv, dtype=np.int32)
    scores = np.zeros((sh.Hkv, max(sh.n_past, 0)), dtype=np.float32)
    d = _desc(sh, bf)
    _lib("f32").oomb_oracle_page_score_topk(ctypes.byref(d), _ptr(q), _ptr(k_pool), _ptr(pt),
                                            ctypes.c_int32(top_k), _ptr(sel), _ptr(cnt), _ptr(scores))
    return sel, cnt, scores


def page_score_topk_cached(sh: Shape, q, kbar_cache, top_k: int):
    """The selection of page_score_topk with the page means read from kbar_cache [>= n_past][Hkv][D]
    float32 (logical page order).  Returns (sel, sel_count, scores)."""
    bf, (q,) = _inputs("f32", q)
    kb = np.ascontiguousarray(kbar_cache, dtype=np.float32)
    assert kb.shape[0] >= sh.n_past and kb.shape[1:] == (sh.Hkv, sh.D)
    sel = np.full((sh.Hkv, top_k + sh.m), -1, dtype=np.int32)
    cnt = np.zeros(sh.Hkv, dtype=np.int32)
    scores = np.zeros((sh.Hkv, max(sh.n_past, 0)), dtype=np.float32)
    d = _desc(sh, bf)
    _lib("f32").oomb_oracle_page_score_topk_cached(ctypes.byref(d), _ptr(q), _ptr(kb), ctypes.c_int32(top_k),
                                                   _ptr(sel), _ptr(cnt), _ptr(scores))
    return sel, cnt, scores


def kv_append(sh: Shape, k_chunk, v_chunk, page_table, k_pool, v_pool, kbar_cache=None):
    """Writes the chunk's K / V [C][Hkv][D] into the m local pages of (copies of) the pools and, if
    kbar_cache [>= n][Hkv][D] float32 is given, the means of those pages into (a copy of) it.
    Returns (k_pool, v_pool, kbar_cache)."""
    bf, (k_chunk, v_chunk, k_pool, v_pool) = _inputs("f32", k_chunk, v_chunk, k_pool, v_pool)
    k_pool, v_pool = k_pool.copy(), v_pool.copy()
    pt = _i32(page_table)
    kb = None if kbar_cache is None else np.ascontiguousarray(kbar_cache, dtype=np.float32).copy()
    d = _desc(sh, bf)
    _lib("f32").oomb_oracle_kv_append(ctypes.byref(d), _ptr(k_chunk), _ptr(v_chunk), _ptr(pt), _ptr(k_pool),
                                      _ptr(v_pool), _ptr(kb) if kb is not None else None)
    return k_pool, v_pool, kb


def page_means(sh: Shape, k_pool, page_table, first: int, count: int, kbar_cache):
    """Means of logical pages [first, first + count) into (a copy of) kbar_cache [..][Hkv][D] float32."""
    bf, (k_pool,) = _inputs("f32", k_pool)
    pt = _i32(page_table)
    kb = np.ascontiguousarray(kbar_cache, dtype=np.float32).copy()
    assert kb.shape[0] >= first + count
    d = _desc(sh, bf)
    _lib("f32").oomb_oracle_page_means(ctypes.byref(d), _ptr(k_pool), _ptr(pt), ctypes.c_int64(first),
                                       ctypes.c_int64(count), _ptr(kb))
    return kb


def page_vote_topk(sh: Shape, q, kbar_cache, top_k: int, kbar_round_bf16=None):
    """Retrieval by voting, one list per (KV head, query page): returns (sel [Hkv][m][top_k + m] int32
    padded with -1, sel_count [Hkv][m], votes [Hkv][m][n_past] float64).  kbar_cache [>= n_past][Hkv][D]
    float32 holds the page means; they are rounded to bf16 first when q is bf16 (or when
    kbar_round_bf16 says so).  Double arithmetic."""
    bf, (q,) = _inputs("f64", q)
    kb = np.ascontiguousarray(kbar_cache, dtype=np.float32)
    assert kb.shape[0] >= sh.n_past and kb.shape[1:] == (sh.Hkv, sh.D)
    rnd = bf if kbar_round_bf16 is None else int(bool(kbar_round_bf16))
    sel = np.full((sh.Hkv, sh.m, top_k + sh.m), -1, dtype=np.int32)
    cnt = np.zeros((sh.Hkv, sh.m), dtype=np.int32)
    votes = np.zeros((sh.Hkv, sh.m, max(sh.n_past, 0)), dtype=np.float64)
    d = _desc(sh, bf)
    _lib("f64").oomb_oracle_page_vote_topk(ctypes.byref(d), _ptr(q), _ptr(kb), ctypes.c_int32(rnd),
                                           ctypes.c_int32(top_k), _ptr(sel), _ptr(cnt), _ptr(votes))
    return sel, cnt, votes


def local_page_list(sh: Shape, window_pages: int):
    """Page list of a local-attention layer: (sel [Hkv][window_pages + m] int32 padded with -1, sel_count)."""
    sel = np.full((sh.Hkv, window_pages + sh.m), -1, dtype=np.int32)
    cnt = np.zeros(sh.Hkv, dtype=np.int32)
    d = _desc(sh, 0)
    _lib("f32").oomb_oracle_local_page_list(ctypes.byref(d), ctypes.c_int32(window_pages), _ptr(sel), _ptr(cnt))
    return sel, cnt


def attn_fwd(sh: Shape, q, k_pool, v_pool, page_table, sel=None, sel_count=None, rows=None,
             prec: str = "f32"):
    """O and LSE.  rows: optional int array [n_rows][2] of (h, i) pairs; then O
    is [n_rows][D] and LSE [n_rows]; otherwise O [C][Hq][D], LSE [Hq][C]."""
    bf, (q, k_pool, v_pool) = _inputs(prec, q, k_pool, v_pool)
    pt = _i32(page_table)
    sel, cnt, stride, qp = _sel_args(sel, sel_count)
    rt = _real(prec)
    if rows is None:
        o = np.zeros((sh.C, sh.Hq, sh.D), dtype=rt)
        lse = np.zeros((sh.Hq, sh.C), dtype=rt)
        nr = 0
    else:
        rows = _i32(rows).reshape(-1, 2)
        nr = rows.shape[0]
        o = np.zeros((nr, sh.D), dtype=rt)
        lse = np.zeros((nr,), dtype=rt)
    d = _desc(sh, bf, qp)
    _lib(prec).oomb_oracle_attn_fwd(ctypes.byref(d), _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(pt),
                                    _ptr(sel), _ptr(cnt), ctypes.c_int32(stride), _ptr(rows),
                                    ctypes.c_int64(nr), _ptr(o), _ptr(lse))
    return o, lse


def row_probs(sh: Shape, q, k_pool, page_table, h: int, i: int, sel=None, sel_count=None,
              prec: str = "f32"):
    """Softmax probabilities of row (h, i) and the token positions they belong to."""
    bf, (q, k_pool) = _inputs(prec, q, k_pool)
    pt = _i32(page_table)
    sel, cnt, stride, qp = _sel_args(sel, sel_count)
    cap = sh.N
    p = np.zeros(cap, dtype=_real(prec))
    tok = np.zeros(cap, dtype=np.int64)
    d = _desc(sh, bf, qp)
    nv = _lib(prec).oomb_oracle_row_probs(ctypes.byref(d), _ptr(q), _ptr(k_pool), _ptr(pt), _ptr(sel),
                                          _ptr(cnt), ctypes.c_int32(stride), ctypes.c_int32(h),
                                          ctypes.c_int32(i), _ptr(p), _ptr(tok))
    return p[:nv].copy(), tok[:nv].copy()


def delta(sh: Shape, d_o, o, prec: str = "f32"):
    """Delta[h][i] = <dO[i,h,:], O[i,h,:]>; O is the oracle's own forward output."""
    bf, (d_o,) = _inputs(prec, d_o)
    o = np.ascontiguousarray(o, dtype=_real(prec))
    out = np.zeros((sh.Hq, sh.C), dtype=_real(prec))
    d = _desc(sh, bf)
    _lib(prec).oomb_oracle_delta(ctypes.byref(d), _ptr(d_o), _ptr(o), _ptr(out))
    return out


def attn_bwd_dq(sh: Shape, q, k_pool, v_pool, page_table, lse, delta_, d_o, sel=None, sel_count=None,
                rows=None, prec: str = "f32"):
    """dQ ([C][Hq][D], or [n_rows][D] for a row subset).  lse/delta_ are [Hq][C]."""
    bf, (q, k_pool, v_pool, d_o) = _inputs(prec, q, k_pool, v_pool, d_o)
    pt = _i32(page_table)
    sel, cnt, stride, qp = _sel_args(sel, sel_count)
    rt = _real(prec)
    lse = np.ascontiguousarray(lse, dtype=rt)
    delta_ = np.ascontiguousarray(delta_, dtype=rt)
    assert lse.shape == (sh.Hq, sh.C) and delta_.shape == (sh.Hq, sh.C)
    if rows is None:
        dq = np.zeros((sh.C, sh.Hq, sh.D), dtype=rt)
        nr = 0
    else:
        rows = _i32(rows).reshape(-1, 2)
        nr = rows.shape[0]
        dq = np.zeros((nr, sh.D), dtype=rt)
    d = _desc(sh, bf, qp)
    _lib(prec).oomb_oracle_attn_bwd_dq(ctypes.byref(d), _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(pt),
                                       _ptr(sel), _ptr(cnt), ctypes.c_int32(stride), _ptr(lse),
                                       _ptr(delta_), _ptr(d_o), _ptr(rows), ctypes.c_int64(nr),
                                       _ptr(dq))
    return dq


def attn_bwd_dkv(sh: Shape, q, k_pool, v_pool, page_table, lse, delta_, d_o, dk_pool, dv_pool,
                 sel=None, sel_count=None, units=None, prec: str = "f32"):
    """Accumulates into dk_pool / dv_pool (arrays of the oracle's arithmetic
    type, shape of the K/V pools) IN PLACE.  units: optional distinct (g, logical
    page) pairs [n_units][2]; default every selected page of every KV head."""
    bf, (q, k_pool, v_pool, d_o) = _inputs(prec, q, k_pool, v_pool, d_o)
    pt = _i32(page_table)
    sel, cnt, stride, qp = _sel_args(sel, sel_count)
    rt = _real(prec)
    lse = np.ascontiguousarray(lse, dtype=rt)
    delta_ = np.ascontiguousarray(delta_, dtype=rt)
    assert dk_pool.dtype == rt and dv_pool.dtype == rt
    assert dk_pool.flags.c_contiguous and dv_pool.flags.c_contiguous
    if units is None:
        nu = 0
    else:
        units = _i32(units).reshape(-1, 2)
        nu = units.shape[0]
        assert len({(int(a), int(b)) for a, b in units}) == nu, "units must be distinct"
    d = _desc(sh, bf, qp)
    _lib(prec).oomb_oracle_attn_bwd_dkv(ctypes.byref(d), _ptr(q), _ptr(k_pool), _ptr(v_pool), _ptr(pt),
                                        _ptr(sel), _ptr(cnt), ctypes.c_int32(stride), _ptr(lse),
                                        _ptr(delta_), _ptr(d_o), _ptr(units), ctypes.c_int64(nu),
                                        _ptr(dk_pool), _ptr(dv_pool))
    return dk_pool, dv_pool


def attn_fwd_bwd(sh: Shape, q, k_pool, v_pool, page_table, d_o, sel=None, sel_count=None,
                 dk_pool=None, dv_pool=None, prec: str = "f32"):
    """Whole pass on all rows: returns dict(o, lse, delta, dq, dk_pool, dv_pool)."""
    rt = _real(prec)
    o, lse = attn_fwd(sh, q, k_pool, v_pool, page_table, sel, sel_count, prec=prec)
    dl = delta(sh, d_o, o, prec=prec)
    dq = attn_bwd_dq(sh, q, k_pool, v_pool, page_table, lse, dl, d_o, sel, sel_count, prec=prec)
    if dk_pool is None:
        dk_pool = np.zeros(k_pool.shape, dtype=rt)
    if dv_pool is None:
        dv_pool = np.zeros(k_pool.shape, dtype=rt)
    attn_bwd_dkv(sh, q, k_pool, v_pool, page_table, lse, dl, d_o, dk_pool, dv_pool, sel, sel_count,
                 prec=prec)
    return dict(o=o, lse=lse, delta=dl, dq=dq, dk_pool=dk_pool, dv_pool=dv_pool)


# ---------------------------------------------------------------------------------------------
# Offloaded KV cache (Sec. 4.3: the KV cache and its gradients live in host memory; the pages a
# chunk attends are brought to the device, the gradients of those pages are taken back).  Pure
# data movement, written as the definition over the page lists themselves:
#   held(g)  = the logical pages in some list of KV head g
#   union    = the pages held by any KV head, ascending
#   slot(l)  = rank of l in union (staging pools are indexed by slot), or "overflow" when the rank is not
#              below the staging capacity
#   fetch:      stage[slot(l)][g]  = host[page_table[l]][g]   for every g and every l in held(g), K and V
#   write-back: host[page_table[l]][g] += stage[slot(l)][g]   for the same (g, l), once each, dK and dV
# Tiles of overflowing pages do not move.  sel is [Hkv][stride] (one list per KV head) or
# [Hkv][m][stride] (one per KV head and query page), sel_count the matching [Hkv] / [Hkv][m].

def _held_pages(sh: Shape, sel, sel_count):
    """held(g) for every KV head, as sorted lists of logical page ids."""
    sel = _i32(sel)
    cnt = _i32(sel_count)
    assert sel.ndim in (2, 3) and cnt.shape == sel.shape[:-1]
    held = []
    for g in range(sh.Hkv):
        lists = sel[g].reshape(-1, sel.shape[-1])
        counts = cnt[g].reshape(-1)
        pages = set()
        for lst, c in zip(lists, counts):
            pages |= set(int(l) for l in lst[:c])
        held.append(sorted(pages))
    return held


def offload_stage_table(sh: Shape, sel, sel_count, capacity=None):
    """The page table of the staging pools: stage_table[l] = slot(l) for the pages of the union, -1 for
    pages in no list; a page whose slot would be >= capacity gets slot 0 (so that the table never points
    outside the staging pools; results are then meaningless and the second return value says so).
    Returns (stage_table [n] int32, number of pages in the union)."""
    held = _held_pages(sh, sel, sel_count)
    union = sorted(set().union(*held)) if held else []
    table = np.full(sh.n, -1, dtype=np.int32)
    for rank, l in enumerate(union):
        table[l] = rank if capacity is None or rank < capacity else 0
    return table, len(union)


def offload_fetch(sh: Shape, host_k, host_v, page_table, sel, sel_count, stage_k, stage_v):
    """Fetch step on copies of the staging pools (capacity = their page count); returns (stage_k, stage_v).
    Nothing but the tiles (slot(l), g) with l in held(g) is written."""
    pt = _i32(page_table)
    stage_k, stage_v = stage_k.copy(), stage_v.copy()
    cap = stage_k.shape[0]
    held = _held_pages(sh, sel, sel_count)
    union = sorted(set().union(*held))
    for g in range(sh.Hkv):
        for l in held[g]:
            s = union.index(l)
            if s < cap:
                stage_k[s, g] = host_k[pt[l], g]
                stage_v[s, g] = host_v[pt[l], g]
    return stage_k, stage_v


def offload_writeback(sh: Shape, stage_dk, stage_dv, host_dk, host_dv, page_table, sel, sel_count):
    """Write-back step on copies of the host gradient pools, in the arithmetic of their dtype (float32 here;
    callers with bf16 pools round the sum); returns (host_dk, host_dv)."""
    pt = _i32(page_table)
    host_dk, host_dv = host_dk.copy(), host_dv.copy()
    cap = stage_dk.shape[0]
    held = _held_pages(sh, sel, sel_count)
    union = sorted(set().union(*held))
    for g in range(sh.Hkv):
        for l in held[g]:
            s = union.index(l)
            if s < cap:
                host_dk[pt[l], g] = host_dk[pt[l], g] + stage_dk[s, g]
                host_dv[pt[l], g] = host_dv[pt[l], g] + stage_dv[s, g]
    return host_dk, host_dv


# ---------------------------------------------------------------------------------------------
# Preconditions of the attention entry points (Sec. 4.1: a page table maps logical pages to distinct
# physical pages; Sec. 4.2: the lists hold the retrieved pages and the chunk's own pages), written
# out as plain checks.  Bits of the result:
CHECK_TABLE_RANGE = 1      # a page-table entry outside [0, n_phys)
CHECK_TABLE_DISTINCT = 2   # two logical pages share a physical page
CHECK_LIST_COUNT = 4       # a list count outside [0, stride]
CHECK_LIST_RANGE = 8       # a list entry outside [0, n)
CHECK_LIST_ORDER = 16      # a list that is not strictly ascending
CHECK_LIST_LOCAL = 32      # a list without the local page(s) it must hold


def check_inputs(sh: Shape, n_phys: int, page_table, sel=None, sel_count=None) -> int:
    """Violations (bit mask) of the documented preconditions.  sel [Hkv][stride] must hold all m local
    pages; sel [Hkv][m][stride] must hold, in the list of query page tau, the local page n_past + tau."""
    pt = _i32(page_table)[: sh.n]
    bad = 0
    in_range = (pt >= 0) & (pt < n_phys)
    if not in_range.all():
        bad |= CHECK_TABLE_RANGE
    ok = pt[in_range]
    if len(np.unique(ok)) != len(ok):
        bad |= CHECK_TABLE_DISTINCT
    if sel is None:
        return bad
    sel, cnt = _i32(sel), _i32(sel_count)
    stride = sel.shape[-1]
    lists = sel.reshape(-1, stride)
    counts = cnt.reshape(-1)
    per_head = lists.shape[0] // sh.Hkv
    for idx, (lst, c) in enumerate(zip(lists, counts)):
        if c < 0 or c > stride:
            bad |= CHECK_LIST_COUNT
            c = min(max(int(c), 0), stride)
        e = lst[:c]
        if ((e < 0) | (e >= sh.n)).any():
            bad |= CHECK_LIST_RANGE
        if (np.diff(e) <= 0).any():
            bad |= CHECK_LIST_ORDER
        need = range(sh.n_past, sh.n) if per_head == 1 else [sh.n_past + idx % per_head]
        if not set(need) <= set(int(v) for v in e):
            bad |= CHECK_LIST_LOCAL
    return bad


class PagePool:
    """Free list of the physical pages shared by the K / V / dK / dV pools (paper Sec. 4.1: pages are handed
    out on demand as the context grows, so nothing is reallocated).  A plain Python list used as a stack:
    after a reset pages come out in ascending order; released pages are reused last-released-first.
    `alloc` raises MemoryError when fewer than `count` pages are free (state unchanged), `release` raises
    ValueError for a page that is out of range, listed twice or already free (state unchanged)."""

    def __init__(self, num_phys_pages: int):
        self.num_phys_pages = int(num_phys_pages)
        self.free = list(range(self.num_phys_pages - 1, -1, -1))   # top of the stack = end of the list

    @property
    def n_free(self) -> int:
        return len(self.free)

    def alloc(self, count: int) -> list:
        if count < 0:
            raise ValueError("negative count")
        if count > len(self.free):
            raise MemoryError("page pool exhausted")
        return [self.free.pop() for _ in range(count)]

    def release(self, pages) -> None:
        pages = [int(x) for x in pages]
        if len(set(pages)) != len(pages) or any(x < 0 or x >= self.num_phys_pages for x in pages) or \
                set(pages) & set(self.free):
            raise ValueError("bad page in release")
        self.free.extend(pages)
