"""Seeded synthetic inputs for the paged sparse attention hot path.

This module only draws random numbers and lays them out; it holds none of the
method's arithmetic and is the one piece shared by the HIP path's tests, the
benchmark and the CPU oracle's tests.

Shapes follow the paper's notation (Sec. 4.2): a chunk of C = m*P query tokens
against N = n*P tokens reachable through the page table, the chunk's own K/V
being the last m logical pages.  The named workloads stand in for the paper's
Qwen2.5-7B runs (28 query heads, 4 KV heads, head dim 128, page size 128,
chunk 4096 / 8192, retrieval budgets of 64 / 128 / 256 pages): only the layer
shape and the page / chunk / budget structure are kept, values are N(0, 1).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Optional

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    Hq: int
    Hkv: int
    D: int
    P: int
    C: int
    N: int                       # tokens reachable through the page table, chunk included
    top_k: Optional[int]         # None = dense (every page selected)
    dtype: str                   # "f32" | "bf16"  (Q, K, V, O, dO, dQ)
    grad_dtype: str              # "f32" | "bf16"  (dK / dV pools)
    sm_scale: float
    q_scale: float = 1.0         # Q = N(0,1) * q_scale
    extra_phys: int = 0          # physical pages beyond n (never referenced)
    boost_frac: float = 0.0      # fraction of past pages whose keys get +boost
    boost: float = 2.0
    boost_run: int = 1           # boosted pages come in runs of this many logical pages
    seed: int = 0

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

    @property
    def n_phys(self) -> int:
        return self.n + self.extra_phys

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


def _qwen(name, C, N, top_k, seed, grad_dtype="f32", **kw):
    return Workload(name=name, Hq=28, Hkv=4, D=128, P=128, C=C, N=N, top_k=top_k, dtype="bf16",
                    grad_dtype=grad_dtype, sm_scale=1.0, q_scale=1.0 / math.sqrt(128.0), seed=seed,
                    **kw)


WORKLOADS = {
    # tiny fp32 case the oracle finishes at once; dense and top-k = 8
    "tiny_dense": Workload("tiny_dense", 2, 1, 64, 16, 128, 1024, None, "f32", "f32", 0.125,
                           extra_phys=5, seed=20260201),
    "tiny_sparse": Workload("tiny_sparse", 2, 1, 64, 16, 128, 1024, 8, "f32", "f32", 0.125,
                            extra_phys=5, boost_frac=0.1, seed=20260201),
    # small bf16 cases on the MFMA kernels (P = 128, D = 128): Qwen-like GQA 7:1, several row
    # tiles with a ragged tail
    "smoke_bf16": Workload("smoke_bf16", 14, 2, 128, 128, 256, 2048, 4, "bf16", "f32", 0.0884,
                           extra_phys=3, boost_frac=0.2, seed=20260210),
    "mid_sparse_bf16": Workload("mid_sparse_bf16", 28, 4, 128, 128, 512, 128 * 24, 6, "bf16", "f32",
                                0.0884, extra_phys=7, boost_frac=0.15, seed=20260211),
    "mid_dense_bf16": Workload("mid_dense_bf16", 6, 2, 128, 128, 384, 128 * 11, None, "bf16", "bf16",
                               0.0884, extra_phys=2, seed=20260212),
    # Qwen2.5-7B-shaped layer, dense over a 64K history
    "qwen_dense_64k": _qwen("qwen_dense_64k", 4096, 65536, None, 20260202),
    # sparse, 256K history, 64 retrieved pages
    "qwen_sparse_256k": _qwen("qwen_sparse_256k", 4096, 262144, 64, 20260203, boost_frac=0.05),
    # sparse, 1M history, 128 retrieved pages (headline); room for 16 chunks of growth
    "qwen_sparse_1m": _qwen("qwen_sparse_1m", 4096, 1048576, 128, 20260204, boost_frac=0.05,
                            extra_phys=480),
    # stress: 4M history, chunk 8192, 256 retrieved pages, clustered boosted pages
    "qwen_sparse_4m": _qwen("qwen_sparse_4m", 8192, 4194304, 256, 20260205, boost_frac=0.05,
                            boost_run=8, grad_dtype="bf16"),
}


def torch_dtype(name: str):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def make_inputs(w: Workload, device="cpu", zero_grad_pools: bool = True) -> dict:
    """Draw every input of one layer/one chunk call.

    Returns tensors on `device`:
      q, d_o       [C][Hq][D]            dtype w.dtype
      k_pool, v_pool [n_phys][Hkv][P][D] dtype w.dtype (logical page l at page_table[l])
      page_table   [n + extra] int32 (a random permutation of the physical pages;
                   entries past n map the spare physical pages, so a growing
                   history can be emulated by raising N)
      dk_pool, dv_pool  like the pools, dtype w.grad_dtype, zeros
      boosted      int64 logical ids of the boosted pages
    """
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed)
    dt = torch_dtype(w.dtype)

    def randn(*shape):
        # drawn in fp32 then rounded, in slabs so the fp32 staging stays small
        out = torch.empty(shape, dtype=dt, device=dev)
        flat = out.view(-1)
        step = 1 << 26
        for s in range(0, flat.numel(), step):
            e = min(flat.numel(), s + step)
            flat[s:e] = torch.randn(e - s, generator=gen, device=dev, dtype=torch.float32).to(dt)
        return out

    q = (randn(w.C, w.Hq, w.D).float() * w.q_scale).to(dt)
    d_o = randn(w.C, w.Hq, w.D)
    k_pool = randn(w.n_phys, w.Hkv, w.P, w.D)
    v_pool = randn(w.n_phys, w.Hkv, w.P, w.D)
    page_table = torch.randperm(w.n_phys, generator=gen, device=dev).to(torch.int32)

    boosted = torch.empty(0, dtype=torch.int64, device=dev)
    if w.boost_frac > 0 and w.n_past > 0:
        n_boost = int(w.boost_frac * w.n_past)
        n_runs = max(1, n_boost // w.boost_run)
        starts = torch.randperm(max(1, w.n_past // w.boost_run), generator=gen, device=dev)[:n_runs]
        ids = (starts[:, None] * w.boost_run + torch.arange(w.boost_run, device=dev)[None, :]).reshape(-1)
        boosted = ids[ids < w.n_past]
        phys = page_table[boosted].long()
        k_pool[phys] = (k_pool[phys].float() + w.boost).to(dt)

    gdt = torch_dtype(w.grad_dtype)
    if zero_grad_pools:
        dk_pool = torch.zeros(k_pool.shape, dtype=gdt, device=dev)
        dv_pool = torch.zeros(k_pool.shape, dtype=gdt, device=dev)
    else:
        dk_pool = dv_pool = None
    return dict(q=q, d_o=d_o, k_pool=k_pool, v_pool=v_pool, page_table=page_table,
                dk_pool=dk_pool, dv_pool=dv_pool, boosted=boosted)


def to_numpy(t: torch.Tensor):
    """Host numpy view of a tensor; bf16 becomes its uint16 bit pattern."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view("uint16")
    return t.numpy()
