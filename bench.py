"""Benchmark of the paged sparse attention hot path on one MI355X.

A step is one pass of the whole hot path over one query chunk of one layer:
page scoring + top-k selection, paged attention forward, paged attention
backward (dQ, dK/dV accumulated into the gradient pool).  The default workload
is the 1M-token-history Qwen2.5-7B-shaped sparse layer; consecutive steps let
the history grow by one chunk (16 chunks, then it wraps), the gradient pools
persisting across steps.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def pairs_of(w, N):
    """Unmasked (query, key) pairs per query head for a chunk ending at N."""
    n_past = N // w.P - w.m
    k_eff = n_past if w.top_k is None else min(w.top_k, n_past)
    return w.C * k_eff * w.P + w.C * (w.C + 1) // 2


def cpu_baseline(w, x, sample_tokens):
    """The CPU oracle, as it stands, on the first `sample_tokens` tokens of the chunk."""
    import numpy as np
    import oracle
    from paper_2602_02108_amd.workloads import to_numpy
    sub = w.with_(C=sample_tokens, N=w.N - w.C + sample_tokens)
    sh = oracle.Shape(sub.Hq, sub.Hkv, sub.D, sub.P, sub.C, sub.N, sub.sm_scale)
    q = to_numpy(x["q"][:sample_tokens])
    d_o = to_numpy(x["d_o"][:sample_tokens])
    k_pool, v_pool, pt = to_numpy(x["k_pool"]), to_numpy(x["v_pool"]), to_numpy(x["page_table"])
    t0 = time.perf_counter()
    sel = cnt = None
    if sub.top_k is not None:
        sel, cnt, _ = oracle.page_score_topk(sh, q, k_pool, pt, sub.top_k)
    t1 = time.perf_counter()
    o, lse = oracle.attn_fwd(sh, q, k_pool, v_pool, pt, sel, cnt)
    dl = oracle.delta(sh, d_o, o)
    dq = oracle.attn_bwd_dq(sh, q, k_pool, v_pool, pt, lse, dl, d_o, sel, cnt)
    # dK/dV pools only for the pages the sample touches (the oracle adds in place)
    dk = np.zeros(k_pool.shape, dtype=np.float32)
    dv = np.zeros(k_pool.shape, dtype=np.float32)
    oracle.attn_bwd_dkv(sh, q, k_pool, v_pool, pt, lse, dl, d_o, dk, dv, sel, cnt)
    t2 = time.perf_counter()
    flops = 14.0 * sub.D * pairs_of(sub, sub.N) * sub.Hq
    return {"value": flops / (t2 - t0) / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"first {sample_tokens} tokens of the chunk, all {sub.Hq} heads, full page scoring "
                      f"({sub.n_past} pages) + top-{sub.top_k} + fwd + bwd; scoring {t1 - t0:.2f} s, "
                      f"attention {t2 - t1:.2f} s",
            "seconds": t2 - t0}


def offload_bench(args, w, x, api, torch, desc_at, top_k, sel, cnt, o, lse, dq, ws_sc, ws_fw, ws_bw, n_max, d_max, votes):
    """Step = cached-means selection -> staging plan -> fetch of the selected pages from pinned host pools ->
    forward + backward on the staging pools -> write-back of the staged gradients into the host pools."""
    dev = x["q"].device
    gdt = x["dk_pool"].dtype
    kbar = torch.zeros((n_max // w.P, w.Hkv, w.D), dtype=torch.float32, device=dev)
    api.page_means(d_max, x["k_pool"], x["page_table"], 0, n_max // w.P, kbar)
    torch.cuda.synchronize()

    def pinned(t, zero=False):
        h = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
        h.zero_() if zero else h.copy_(t)
        return h

    host_k, host_v = pinned(x["k_pool"]), pinned(x["v_pool"])
    host_dk, host_dv = pinned(x["dk_pool"], True), pinned(x["dv_pool"], True)
    stride = top_k + w.m
    cap = min(n_max // w.P, sel.numel())
    select = (lambda desc, s_, c_: api.page_vote_topk(desc, x["q"], kbar, top_k, s_, c_, workspace=ws_sc)) if votes else \
        (lambda desc, s_, c_: api.page_score_topk_cached(desc, x["q"], kbar, top_k, s_, c_, workspace=ws_sc))
    fwd = api.paged_attn_fwd_qp if votes else api.paged_attn_fwd
    bwd = api.paged_attn_bwd_qp if votes else api.paged_attn_bwd
    shape = (cap,) + tuple(x["k_pool"].shape[1:])
    bufs = [dict(k=torch.empty(shape, dtype=x["k_pool"].dtype, device=dev), v=torch.empty(shape, dtype=x["k_pool"].dtype, device=dev),
                 dk=torch.empty(shape, dtype=gdt, device=dev), dv=torch.empty(shape, dtype=gdt, device=dev),
                 sel=torch.empty_like(sel), cnt=torch.empty_like(cnt), plan=api.OffloadPlan(d_max, cap, dev))
            for _ in range(3)]
    main = torch.cuda.current_stream()
    copy = torch.cuda.Stream()

    def resident(s):
        N, desc = desc_at(s)
        select(desc, sel, cnt)
        fwd(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], sel, cnt, o, lse, ws_fw)
        bwd(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], o, lse, x["d_o"], x["dk_pool"], x["dv_pool"],
            sel, cnt, dq, ws_bw)

    def select_plan(s, b):
        N, desc = desc_at(s)
        select(desc, b["sel"], b["cnt"])
        api.offload_plan(desc, b["sel"], b["cnt"], b["plan"])   # plan.stage_table = page table of the staging pools

    def fetch(s, b, stream):
        N, desc = desc_at(s)
        api.offload_fetch(desc, host_k, host_v, x["page_table"], b["plan"], b["k"], b["v"], b["dk"], b["dv"], stream=stream)

    def attend(s, b):
        N, desc = desc_at(s)
        pt = b["plan"].stage_table
        fwd(desc, x["q"], b["k"], b["v"], pt, b["sel"], b["cnt"], o, lse, ws_fw)
        bwd(desc, x["q"], b["k"], b["v"], pt, o, lse, x["d_o"], b["dk"], b["dv"], b["sel"], b["cnt"], dq, ws_bw)

    def writeback(s, b, stream):
        N, desc = desc_at(s)
        api.offload_writeback(desc, b["dk"], b["dv"], host_dk, host_dv, x["page_table"], b["plan"], stream=stream)

    def serial(s):
        b = bufs[0]
        select_plan(s, b)
        fetch(s, b, None)
        attend(s, b)
        writeback(s, b, None)

    def overlapped(K):
        # The fetch of step s + 1 and the write-back of step s - 1 run on the copy stream while step s computes.
        # Three buffer sets: the copy stream runs fetch(s), wb(s - 1), fetch(s + 1), wb(s), ... in that order, and the
        # main stream touches set (s + 1) % 3 only after fetch(s) has landed, i.e. after wb(s - 2), its last user.
        ev = lambda: torch.cuda.Event()
        select_plan(0, bufs[0])
        e = ev(); e.record(main); copy.wait_event(e)
        fetch(0, bufs[0], copy)
        fetched = ev(); fetched.record(copy)
        for s in range(K):
            b = bufs[s % 3]
            main.wait_event(fetched)
            if s + 1 < K:
                nb = bufs[(s + 1) % 3]
                select_plan(s + 1, nb)
                e = ev(); e.record(main); copy.wait_event(e)
                fetch(s + 1, nb, copy)
                fetched = ev(); fetched.record(copy)
            attend(s, b)
            e = ev(); e.record(main); copy.wait_event(e)
            writeback(s, b, copy)
        e = ev(); e.record(copy); main.wait_event(e)

    def timed(fn):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    K = args.steps
    for s in range(args.warmup):
        resident(s); serial(s)
    overlapped(2)
    ms_res = timed(lambda: [resident(s) for s in range(K)])
    ms_ser = timed(lambda: [serial(s) for s in range(K)])
    ms_ovl = timed(lambda: overlapped(K))
    api.profile_reset(); api.profile_enable(1)
    for s in range(K):
        serial(s)
    torch.cuda.synchronize()
    api.profile_enable(False)
    prof = {k: v[0] / max(v[1], 1) for k, v in api.profile_read().items()}
    flops = sum(14.0 * w.D * pairs_of(w, desc_at(s)[0]) * w.Hq for s in range(K))
    es = x["k_pool"].element_size()
    # (page, KV head) tiles moved by the last step: the set bits of the plan's head mask
    n_last = desc_at(K - 1)[0] // w.P   # (the plan of the last serial step covers its own n pages only)
    mask = bufs[0]["plan"].head_mask.cpu().numpy().view("uint32")[:n_last]
    tiles = int(sum(bin(int(v)).count("1") for v in mask[mask != 0]))
    fetch_bytes = tiles * 2 * w.P * w.D * es
    wb_bytes = tiles * 2 * w.P * w.D * x["dk_pool"].element_size() * 2   # host read + host write
    exposed = max(ms_ser - ms_res, 1e-9)
    return {
        "metric": "paged sparse attn fwd+bwd TFLOP/s per layer at 1M-token history, KV cache and gradients offloaded",
        "value": flops / (ms_ovl * 1e-3 * K) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": ms_ovl, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "offload": "K/V and dK/dV pools in pinned host memory; selected pages staged",
                   "top_k_pages": top_k, "local_pages": w.m, "scoring": "cached page means",
                   "retrieval": "softmax votes, one list per query page" if votes else
                                "pooled query score, one list per KV head", "tiles_moved_per_step": tiles},
        "offload": {"ms_per_step_resident": ms_res, "ms_per_step_serial": ms_ser, "ms_per_step_overlapped": ms_ovl,
                    "overhead_serial": ms_ser / ms_res - 1.0, "overhead_overlapped": ms_ovl / ms_res - 1.0,
                    "overlap_fraction": (ms_ser - ms_ovl) / exposed,
                    "fetch_ms": prof.get("offload_fetch"), "writeback_ms": prof.get("offload_writeback"),
                    "plan_ms": prof.get("offload_plan"),
                    "fetch_bytes": fetch_bytes, "writeback_link_bytes": wb_bytes,
                    "fetch_GBps": fetch_bytes / (prof["offload_fetch"] * 1e-3) / 1e9 if prof.get("offload_fetch") else None,
                    "writeback_GBps": wb_bytes / (prof["offload_writeback"] * 1e-3) / 1e9 if prof.get("offload_writeback") else None},
        "kernels_ms": prof,
    }


def quick_measure(api, torch, name, steps, warmup):
    """One of the other benchmark configurations, outside the headline's timed region: `warmup` untimed steps, then
    `steps` steps (streaming scorer, pooled retrieval, history fixed at the configuration's N) timed as a whole with
    the three large attention kernels and the page scorer bracketed by events.  Returns the step time, the
    credited TFLOP/s and the dominant kernel's roofline fraction."""
    from paper_2602_02108_amd.workloads import WORKLOADS, make_inputs, torch_dtype
    w = WORKLOADS[name]
    dev = torch.device("cuda:0")
    x = make_inputs(w, dev)
    desc = api.make_desc(x["q"], x["k_pool"], w.N, w.sm_scale, torch_dtype(w.grad_dtype))
    k = w.top_k
    lk = k if k is not None else -1
    ws_sc = torch.empty(max(api.workspace_bytes(desc, k or 0, api.OP_SCORE_TOPK), 256), dtype=torch.uint8, device=dev)
    ws_fw = torch.empty(api.workspace_bytes(desc, lk, api.OP_ATTN_FWD), dtype=torch.uint8, device=dev)
    ws_bw = torch.empty(api.workspace_bytes(desc, lk, api.OP_ATTN_BWD), dtype=torch.uint8, device=dev)
    sel = torch.empty((w.Hkv, (k or 0) + w.m), dtype=torch.int32, device=dev)
    cnt = torch.empty((w.Hkv,), dtype=torch.int32, device=dev)
    o, dq = torch.empty_like(x["q"]), torch.empty_like(x["q"])
    lse = torch.empty((w.Hq, w.C), dtype=torch.float32, device=dev)

    def step():
        sl = ct = None
        if k is not None:
            api.page_score_topk(desc, x["q"], x["k_pool"], x["page_table"], k, sel, cnt, workspace=ws_sc)
            sl, ct = sel, cnt
        api.paged_attn_fwd(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], sl, ct, o, lse, ws_fw)
        api.paged_attn_bwd(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], o, lse, x["d_o"], x["dk_pool"],
                           x["dv_pool"], sl, ct, dq, ws_bw)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    api.profile_reset()
    api.profile_enable(2)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    api.profile_enable(False)
    prof = api.profile_read()
    api.profile_reset()
    pairs = pairs_of(w, w.N)
    flops = 14.0 * w.D * pairs * w.Hq
    kern = {kn: v[0] / max(v[1], 1) for kn, v in prof.items()}
    credited = {"attn_fwd_mfma": 4.0, "bwd_dq_mfma": 6.0, "bwd_dkv_mfma": 4.0}
    dom = max(kern, key=kern.get)
    out = {"ms_per_step": dt * 1e3 / steps, "steps": steps, "warmup": warmup, "tflops": flops * steps / dt / 1e12,
           "frac_mfma_peak": flops * steps / dt / 1e12 / MFMA_BF16_PEAK_TFLOPS,
           "tflop_per_step": flops / 1e12, "history_tokens": w.N, "chunk": w.C, "top_k_pages": w.top_k,
           "grad_pool_dtype": w.grad_dtype, "kernels_ms": kern, "dominant_kernel": dom}
    if dom in credited:
        ach = credited[dom] * w.D * pairs * w.Hq / (kern[dom] * 1e-3) / 1e12
        out["dominant_kernel_roofline"] = {"bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS,
                                           "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS}
    if "page_score" in kern:
        gbs = w.n_past * w.P * w.D * 2 * w.Hkv / (kern["page_score"] * 1e-3) / 1e9
        out["page_score_GBps"] = gbs
        out["page_score_frac_hbm_peak"] = gbs / HBM_PEAK_GBS
    return out


def quick_votes(api, torch, w, x, steps, warmup):
    """The headline workload with the paper's own retrieval rule (Sec. 4.2 scoring equation: softmax votes summed
    per query page, one list per query page; cached page means), a few steps outside the headline's timed
    region: step time, credited TFLOP/s and the per-kernel times."""
    dev = x["q"].device
    from paper_2602_02108_amd.workloads import torch_dtype
    desc = api.make_desc(x["q"], x["k_pool"], w.N, w.sm_scale, torch_dtype(w.grad_dtype))
    k = w.top_k
    kbar = torch.zeros((w.n, w.Hkv, w.D), dtype=torch.float32, device=dev)
    api.page_means(desc, x["k_pool"], x["page_table"], 0, w.n, kbar)
    ws_sc = torch.empty(api.workspace_bytes(desc, k, api.OP_VOTE_TOPK), dtype=torch.uint8, device=dev)
    ws_fw = torch.empty(api.workspace_bytes(desc, k, api.OP_ATTN_FWD_QP), dtype=torch.uint8, device=dev)
    ws_bw = torch.empty(api.workspace_bytes(desc, k, api.OP_ATTN_BWD_QP), dtype=torch.uint8, device=dev)
    sel = torch.empty((w.Hkv, w.m, k + w.m), dtype=torch.int32, device=dev)
    cnt = torch.empty((w.Hkv, w.m), dtype=torch.int32, device=dev)
    o, dq = torch.empty_like(x["q"]), torch.empty_like(x["q"])
    lse = torch.empty((w.Hq, w.C), dtype=torch.float32, device=dev)

    def step():
        api.page_vote_topk(desc, x["q"], kbar, k, sel, cnt, workspace=ws_sc)
        api.paged_attn_fwd_qp(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], sel, cnt, o, lse, ws_fw)
        api.paged_attn_bwd_qp(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], o, lse, x["d_o"], x["dk_pool"],
                              x["dv_pool"], sel, cnt, dq, ws_bw)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    api.profile_reset()
    api.profile_enable(1)
    for _ in range(2):
        step()
    torch.cuda.synchronize()
    api.profile_enable(False)
    kern = {kn: v[0] / max(v[1], 1) for kn, v in api.profile_read().items()}
    api.profile_reset()
    # every query page keeps top_k past pages of its own: the same pair count as one list per KV head
    flops = 14.0 * w.D * pairs_of(w, w.N) * w.Hq
    return {"retrieval": "softmax votes, one list per query page; cached page means", "ms_per_step": dt * 1e3 / steps,
            "steps": steps, "warmup": warmup, "tflops": flops * steps / dt / 1e12,
            "frac_mfma_peak": flops * steps / dt / 1e12 / MFMA_BF16_PEAK_TFLOPS, "kernels_ms": kern}


def rocminfo_max_clock_mhz():
    """Max shader clock of the first GPU agent as rocminfo prints it (None if it cannot be read)."""
    try:
        import subprocess
        txt = subprocess.run(["rocminfo"], capture_output=True, text=True, timeout=20).stdout
        gpu = txt.split("Device Type:             GPU")
        if len(gpu) < 2:
            return None
        # the clock line precedes "Device Type" inside the agent block: search the block of that agent
        block = txt[txt.rfind("*******", 0, txt.find("Device Type:             GPU")):]
        for line in block.splitlines():
            if "Max Clock Freq. (MHz)" in line:
                return int(line.split(":")[1].strip())
    except Exception:
        return None
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=16)
    ap.add_argument("--warmup", type=int, default=16,
                    help="untimed steps before the timed ones (default: one pass over the 16-chunk sequence, after which\n"
                         "the step time is steady; with 4 the first timed chunks still run 3 %% slower)")
    ap.add_argument("--workload", default="qwen_sparse_1m")
    ap.add_argument("--cpu-sample-tokens", type=int, default=1024)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cached-means", action="store_true",
                    help="score the pages from cached page means (kept by the paged manager at append time) "
                         "instead of streaming every past key; the default is the streaming scorer")
    ap.add_argument("--retrieval", choices=["pooled", "votes"], default="pooled",
                    help="pooled: one score per key page from the mean-pooled chunk query, one page list per KV head "
                         "(the benchmark configuration); votes: per-token softmax votes summed per query page, one "
                         "list per query page (the paper's scoring equation)")
    ap.add_argument("--offload", action="store_true",
                    help="keep the K / V pools and their gradient pools in pinned host memory: every step fetches the "
                         "selected pages into device staging pools and adds their gradients back (pooled retrieval, "
                         "cached page means); reports the step time without offload, with the transfers serialised, "
                         "and with the transfers on a second stream overlapping the neighbouring steps")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short runs of the other benchmark configurations (dense 64K, sparse 256K, sparse 4M) "
                         "that the default run appends as `other_workloads`")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy (a reference for scaling HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2602_02108_amd import api
    from paper_2602_02108_amd.workloads import WORKLOADS, make_inputs, torch_dtype
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    api.lib()  # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    w = WORKLOADS[args.workload]
    x = make_inputs(w, dev)
    grow = w.extra_phys // w.m + 1          # chunks the pre-filled pool can hold
    gdt = torch_dtype(w.grad_dtype)

    def desc_at(step):
        N = w.N + (step % grow) * w.C
        return N, api.make_desc(x["q"], x["k_pool"], N, w.sm_scale, gdt)

    top_k = w.top_k
    votes = args.retrieval == "votes"
    assert not votes or top_k is not None, "--retrieval votes needs a sparse workload"
    n_max, d_max = desc_at(grow - 1)
    ws_sc = torch.empty(max(api.workspace_bytes(d_max, top_k or 0, api.OP_SCORE_TOPK), 256), dtype=torch.uint8, device=dev)
    ws_fw = torch.empty(api.workspace_bytes(d_max, top_k if top_k is not None else -1, api.OP_ATTN_FWD), dtype=torch.uint8,
                        device=dev)
    ws_bw = torch.empty(api.workspace_bytes(d_max, top_k if top_k is not None else -1, api.OP_ATTN_BWD), dtype=torch.uint8,
                        device=dev)
    sel = torch.empty((w.Hkv, (top_k or 0) + w.m), dtype=torch.int32, device=dev)
    cnt = torch.empty((w.Hkv,), dtype=torch.int32, device=dev)
    o = torch.empty_like(x["q"])
    lse = torch.empty((w.Hq, w.C), dtype=torch.float32, device=dev)
    dq = torch.empty_like(x["q"])

    if votes:
        ws_sc = torch.empty(api.workspace_bytes(d_max, top_k, api.OP_VOTE_TOPK), dtype=torch.uint8, device=dev)
        ws_fw = torch.empty(api.workspace_bytes(d_max, top_k, api.OP_ATTN_FWD_QP), dtype=torch.uint8, device=dev)
        ws_bw = torch.empty(api.workspace_bytes(d_max, top_k, api.OP_ATTN_BWD_QP), dtype=torch.uint8, device=dev)
        sel = torch.empty((w.Hkv, w.m, top_k + w.m), dtype=torch.int32, device=dev)
        cnt = torch.empty((w.Hkv, w.m), dtype=torch.int32, device=dev)

    kbar_cache = None
    if votes and not args.cached_means:
        kbar_stream = torch.zeros((n_max // w.P, w.Hkv, w.D), dtype=torch.float32, device=dev)
    if args.cached_means and top_k is not None:
        # the pool is pre-filled; its page means are what the manager would have cached append by append
        kbar_cache = torch.zeros((n_max // w.P, w.Hkv, w.D), dtype=torch.float32, device=dev)
        api.page_means(d_max, x["k_pool"], x["page_table"], 0, n_max // w.P, kbar_cache)

    def step_votes(s):
        N, desc = desc_at(s)
        if kbar_cache is not None:
            kb = kbar_cache
        else:  # the page means are taken from the keys every chunk, as the method is written
            kb = kbar_stream
            api.page_means(desc, x["k_pool"], x["page_table"], 0, N // w.P - w.m, kb)
        api.page_vote_topk(desc, x["q"], kb, top_k, sel, cnt, workspace=ws_sc)
        api.paged_attn_fwd_qp(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], sel, cnt, o, lse, ws_fw)
        api.paged_attn_bwd_qp(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], o, lse, x["d_o"],
                              x["dk_pool"], x["dv_pool"], sel, cnt, dq, ws_bw)
        return N

    def step(s):
        if votes:
            return step_votes(s)
        N, desc = desc_at(s)
        if top_k is not None:
            if kbar_cache is not None:
                api.page_score_topk_cached(desc, x["q"], kbar_cache, top_k, sel, cnt, workspace=ws_sc)
            else:
                api.page_score_topk(desc, x["q"], x["k_pool"], x["page_table"], top_k, sel, cnt, workspace=ws_sc)
            sl, ct = sel, cnt
        else:
            sl = ct = None
        api.paged_attn_fwd(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], sl, ct, o, lse, ws_fw)
        api.paged_attn_bwd(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], o, lse, x["d_o"],
                           x["dk_pool"], x["dv_pool"], sl, ct, dq, ws_bw)
        return N

    if args.offload:
        assert top_k is not None, "--offload needs a sparse workload"
        off = offload_bench(args, w, x, api, torch, desc_at, top_k, sel, cnt, o, lse, dq, ws_sc, ws_fw, ws_bw, n_max, d_max,
                            votes)
        print(json.dumps(off))
        return

    if args.calibrate_copy:
        # an elementwise kernel (not a DMA copy) that reads 1 GiB and writes 1 GiB
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst
    for s in range(args.warmup):
        step(s)
    torch.cuda.synchronize()
    api.profile_reset()
    api.profile_enable(2)   # the timed region brackets only the four large kernels with events
    flops = 0.0
    kv_bytes = 0.0
    pairs_sum = 0
    chunk_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        chunk_ev[s][0].record()
        N = step(s)
        chunk_ev[s][1].record()
        pr = pairs_of(w, N)
        pairs_sum += pr
        flops += 14.0 * w.D * pr * w.Hq
        n_past = N // w.P - w.m
        k_eff = n_past if top_k is None else min(top_k, n_past)
        page_bytes = w.P * w.D * 2 * w.Hkv
        grad_bytes = w.P * w.D * (2 if w.grad_dtype == "bf16" else 4) * w.Hkv
        scored = n_past * page_bytes if top_k is not None else 0
        # K scored once + K,V gathered by forward + dK,dV pages read and written by backward
        kv_bytes += scored + 2 * (k_eff + w.m) * page_bytes + 2 * 2 * (k_eff + w.m) * grad_bytes
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    api.profile_enable(False)
    prof = api.profile_read()
    dt = t1 - t0
    # one more pass of the same steps with every kernel bracketed, for the full per-kernel table
    api.profile_reset()
    api.profile_enable(1)
    for s in range(args.steps):
        step(s)
    torch.cuda.synchronize()
    api.profile_enable(False)
    prof_all = api.profile_read()
    per_chunk_ms = [a.elapsed_time(b) for a, b in chunk_ev]
    # the same K-step sequence twice more (per-kernel timing off, gradient pools restored to zero
    # in between): run-to-run spread and the minimum; `value` stays the first, contract-timed run
    repeats_ms = [dt * 1e3 / args.steps]
    for _ in range(2):
        if x["dk_pool"] is not None:
            x["dk_pool"].zero_()
            x["dv_pool"].zero_()
        torch.cuda.synchronize()
        r0 = time.perf_counter()
        for s in range(args.steps):
            step(s)
        torch.cuda.synchronize()
        repeats_ms.append((time.perf_counter() - r0) * 1e3 / args.steps)

    # dominant kernel and its roofline
    name, (ms_tot, launches) = max(prof.items(), key=lambda kv: kv[1][0])
    avg_ms = ms_tot / max(launches, 1)
    pairs_avg = pairs_sum / args.steps
    credited = {"attn_fwd_mfma": 4.0, "bwd_dq_mfma": 6.0, "bwd_dkv_mfma": 4.0}  # x D x pairs x Hq, algorithmic
    if name in credited:
        ach = credited[name] * w.D * pairs_avg * w.Hq / (avg_ms * 1e-3) / 1e12
        roof = {"kernel": name, "bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": None, "avg_ms": avg_ms, "launches": launches}
    else:
        n_past = w.n_past
        by = n_past * w.P * w.D * 2 * w.Hkv
        ach = by / (avg_ms * 1e-3) / 1e9
        roof = {"kernel": name, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": ach / HBM_PEAK_GBS, "traffic": None, "avg_ms": avg_ms, "launches": launches}
    # HBM traffic of the dominant kernel (bytes per launch, read + write) from the committed
    # FETCH_SIZE / WRITE_SIZE profile of this workload, if there is one
    tpath = os.path.join(ROOT, "profiles", f"hbm_traffic_{w.name}.txt")
    if os.path.exists(tpath):
        for line in open(tpath):
            f = line.split()
            if len(f) == 5 and f[0] == name and f[1] == "read_bytes" and f[3] == "write_bytes":
                roof["traffic"] = int(f[2]) + int(f[4])
                roof["traffic_source"] = (f"profiles/hbm_traffic_{w.name}.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of "
                                          "this command, replayed from the committed summary, not measured in this run")
    # matrix-pipe utilisation of the dominant kernel by hardware counters (busy cycles of the matrix pipes over
    # 4 SIMDs x busy cycles of the compute units), from the committed SQ counter profile of this workload
    upath = os.path.join(ROOT, "profiles", f"mfma_utilisation_{w.name}.txt")
    if roof["bound"] == "mfma" and os.path.exists(upath):
        for line in open(upath):
            f = line.split()
            if len(f) == 7 and f[0] == name and f[5] == "utilisation":
                roof["mfma_utilisation_by_counters"] = float(f[6])
                roof["mfma_utilisation_source"] = (f"profiles/mfma_utilisation_{w.name}.txt: rocprofv3 --pmc SQ counter run of "
                                                   "this command, replayed from the committed summary, not measured in this run")
    kernels = {k: {"avg_ms": v[0] / max(v[1], 1), "launches": v[1]} for k, v in prof_all.items()}
    for k, v in prof.items():  # the large kernels: durations of the timed region itself
        kernels[k] = {"avg_ms": v[0] / max(v[1], 1), "launches": v[1]}
    # measured ceilings of this device (outside the timed region): an MFMA issue loop and a streaming copy
    cbuf = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    ceil_mfma = api.calibrate(0, cbuf)
    ceil_mfma_random = api.calibrate(2, cbuf)   # same loop on random operands: the clock follows the switching activity
    ceil_copy = api.calibrate(1, cbuf)
    del cbuf
    props = torch.cuda.get_device_properties(0)
    roof["measured_ceiling"] = ceil_mfma if roof["bound"] == "mfma" else ceil_copy
    roof["frac_of_measured_ceiling"] = roof["achieved"] / roof["measured_ceiling"]
    if roof["bound"] == "mfma":
        roof["measured_ceiling_random_operands"] = ceil_mfma_random
        roof["frac_of_measured_ceiling_random_operands"] = roof["achieved"] / ceil_mfma_random
    # per phase: algorithmic FLOPs over the summed kernel times of the phase
    def phase_ms(names):
        return sum(kernels[k]["avg_ms"] * kernels[k]["launches"] for k in names if k in kernels) / args.steps
    # (kv_layout belongs to the forward; qp_prepare runs once per phase)
    fwd_ms = phase_ms(["kv_layout", "qp_prepare", "attn_fwd_mfma"]) - 0.5 * phase_ms(["qp_prepare"])
    bwd_ms = phase_ms(["bwd_prep", "bwd_dq_mfma", "bwd_dkv_mfma", "bwd_dkv_reduce"]) + 0.5 * phase_ms(["qp_prepare"])
    sel_ms = phase_ms(["qpool_partial", "qpool_final", "page_score", "page_score_cached", "topk_select", "page_means",
                       "kbar_image", "vote_lse", "vote_sum", "vote_finish"])
    phases = {"select_ms": sel_ms, "fwd_ms": fwd_ms, "bwd_ms": bwd_ms,
              "fwd_tflops": 4.0 * w.D * pairs_avg * w.Hq / (fwd_ms * 1e-3) / 1e12 if fwd_ms > 0 else None,
              "bwd_tflops": 10.0 * w.D * pairs_avg * w.Hq / (bwd_ms * 1e-3) / 1e12 if bwd_ms > 0 else None}
    if "page_score" in kernels:
        by = sum((desc_at(s)[0] // w.P - w.m) for s in range(args.steps)) / args.steps * w.P * w.D * 2 * w.Hkv
        kernels["page_score"]["GB/s"] = by / (kernels["page_score"]["avg_ms"] * 1e-3) / 1e9
        kernels["page_score"]["frac_hbm_peak"] = kernels["page_score"]["GB/s"] / HBM_PEAK_GBS

    out = {
        "metric": "paged sparse attn fwd+bwd TFLOP/s and KV GB/s per layer at 1M-token history",
        "value": flops / dt / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "q_heads": w.Hq, "kv_heads": w.Hkv, "head_dim": w.D, "page_size": w.P,
                   "chunk": w.C, "history_tokens_first_step": w.N, "history_growth_per_step": w.C,
                   "top_k_pages": w.top_k, "local_pages": w.m, "grad_pool_dtype": w.grad_dtype,
                   "scoring": "cached page means" if kbar_cache is not None else "streams every past key",
                   "retrieval": "softmax votes, one list per query page" if votes else
                                "pooled query score, one list per KV head"},
        "kv_gbps": kv_bytes / dt / 1e9,
        "frac_mfma_peak": flops / dt / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "kernels": kernels,
        "phases": phases,
        "ms_per_step_runs": repeats_ms, "ms_per_step_min": min(repeats_ms), "ms_per_chunk": per_chunk_ms,
        "device": {"name": props.name, "compute_units": props.multi_processor_count,
                   "max_clock_mhz": rocminfo_max_clock_mhz()},
        "ceilings": {"mfma_bf16_tflops_measured": ceil_mfma, "mfma_bf16_tflops_measured_random_operands": ceil_mfma_random,
                     "copy_gbs_measured": ceil_copy,
                     "mfma_bf16_tflops_peak": MFMA_BF16_PEAK_TFLOPS, "hbm_gbs_peak": HBM_PEAK_GBS,
                     "value_frac_of_measured_mfma": flops / dt / 1e12 / ceil_mfma,
                     "value_frac_of_measured_mfma_random_operands": flops / dt / 1e12 / ceil_mfma_random},
        "roofline": roof,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, x, args.cpu_sample_tokens)
    plain = args.workload == "qwen_sparse_1m" and not votes and kbar_cache is None
    if plain and not args.no_other_workloads:
        # the same workload in the two widened modes, a few steps each
        modes = {"votes": quick_votes(api, torch, w, x, 6, 2)}
        import types
        oa = types.SimpleNamespace(steps=6, warmup=2)
        x["dk_pool"].zero_(); x["dv_pool"].zero_()
        off = offload_bench(oa, w, x, api, torch, desc_at, top_k, sel, cnt, o, lse, dq, ws_sc, ws_fw, ws_bw, n_max, d_max, False)
        modes["offload"] = {"retrieval": "pooled query score, one list per KV head; cached page means",
                            "ms_per_step": off["ms_per_step"], "steps": 6, "warmup": 2, "tflops": off["value"],
                            **off["offload"]}
        out["other_modes_qwen_sparse_1m"] = modes
        # the other benchmark configurations, a few steps each, after the headline's buffers are gone
        del x, ws_sc, ws_fw, ws_bw, o, dq, lse, sel, cnt
        torch.cuda.empty_cache()
        others = {}
        free, _ = torch.cuda.mem_get_info()
        for name_, steps_ in (("qwen_dense_64k", 6), ("qwen_sparse_256k", 8), ("qwen_sparse_4m", 6)):
            if name_ == "qwen_sparse_4m" and free < 48 * 2**30:
                others[name_] = {"skipped": "needs about 40 GiB of free device memory"}
                continue
            others[name_] = quick_measure(api, torch, name_, steps_, 3)
            torch.cuda.empty_cache()
        out["other_workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
