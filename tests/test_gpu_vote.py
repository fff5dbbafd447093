"""GPU parity of the retrieval by voting (paper Sec. 4.2, the scoring equation: softmax over the key
pages per query token, summed per query page, top-K per query page) against the CPU oracle, and of
the whole per-query-page path (votes -> lists -> attention forward / backward).

The votes are floating point (fp32 on the GPU, double in the oracle) and decide integers (the
lists).  Both sides take the page means in the same precision (bf16 for bf16 tensors); the votes are
compared with a tolerance, and a list is accepted if it is the oracle's list or differs from it
only in pages whose oracle votes tie with the k-th largest vote within that tolerance."""
import numpy as np
import pytest
import torch

from paper_2602_02108_amd import api
from paper_2602_02108_amd.workloads import WORKLOADS, Workload, make_inputs, torch_dtype

import oracle as orc
import parity_util as pu
from test_gpu_qp_attention import gpu_fwd_bwd_qp

pytestmark = pytest.mark.gpu

VOTE_RTOL = 2e-4   # fp32 sums of up to G * P terms and exp2 / log2 of the hardware against double arithmetic


def gpu_means(w, x):
    desc = api.make_desc(x["q"], x["k_pool"], w.N, w.sm_scale, torch_dtype(w.grad_dtype))
    cache = torch.zeros((w.n, w.Hkv, w.D), dtype=torch.float32, device="cuda")
    api.page_means(desc, x["k_pool"], x["page_table"], 0, w.n, cache)
    return desc, cache


def gpu_vote(w, x, top_k):
    desc, cache = gpu_means(w, x)
    votes = torch.zeros((w.Hkv, w.m, max(w.n_past, 1)), dtype=torch.float32, device="cuda")
    sel, cnt = api.page_vote_topk(desc, x["q"], cache, top_k, votes_out=votes)
    torch.cuda.synchronize()
    return sel.cpu().numpy(), cnt.cpu().numpy(), votes[:, :, : w.n_past].cpu().numpy(), cache.cpu().numpy()


def check_lists(w, top_k, sel, cnt, osel, ocnt, ovotes, rtol=VOTE_RTOL):
    """Every list: right length, ascending, the visible local pages at its end, and its past pages are
    a valid top-k of the oracle's votes up to ties within rtol.  Returns the number of lists that are
    not identical to the oracle's."""
    k_eff = min(top_k, w.n_past)
    differ = 0
    assert sel.shape == (w.Hkv, w.m, top_k + w.m)
    for g in range(w.Hkv):
        for tau in range(w.m):
            c = int(cnt[g, tau])
            assert c == k_eff + tau + 1 == int(ocnt[g, tau])
            lst = sel[g, tau, :c]
            assert (np.diff(lst) > 0).all() and (sel[g, tau, c:] == -1).all()
            assert list(lst[k_eff:]) == list(range(w.n_past, w.n_past + tau + 1))
            if np.array_equal(sel[g, tau], osel[g, tau]):
                continue
            differ += 1
            past = lst[:k_eff]
            v = ovotes[g, tau]
            vk = np.sort(v)[::-1][k_eff - 1]
            dropped = np.setdiff1d(np.arange(w.n_past), past)
            assert v[past].min() >= vk * (1 - rtol), (g, tau, v[past].min(), vk)
            assert v[dropped].max() <= vk * (1 + rtol), (g, tau, v[dropped].max(), vk)
    return differ


def vote_parity(w: Workload, top_k: int):
    x = make_inputs(w, "cuda")
    hx = pu.host_inputs(x)
    sel, cnt, votes, cache = gpu_vote(w, x, top_k)
    sh = pu.shape_of(w)
    okb = orc.page_means(sh, hx["k_pool"], hx["page_table"], 0, w.n, np.zeros((w.n, w.Hkv, w.D), np.float32))
    assert np.array_equal(cache.view(np.uint32), okb.view(np.uint32)), "page means differ"
    osel, ocnt, ovotes = orc.page_vote_topk(sh, hx["q"], okb, top_k)
    if w.n_past > 0:
        err = np.abs(votes - ovotes) / np.maximum(ovotes, 1e-30)
        rel = np.linalg.norm(votes - ovotes) / np.linalg.norm(ovotes)
        print(w.name, f"votes: max rel {err.max():.2e}, rel-L2 {rel:.2e}", flush=True)
        assert err.max() < VOTE_RTOL and rel < 2e-5
        assert np.allclose(votes.sum(axis=2), w.P * w.G, rtol=1e-4)
    differ = check_lists(w, top_k, sel, cnt, osel, ocnt, ovotes)
    return x, hx, sel, cnt, osel, ocnt, differ


VOTE_CASES = [
    # matrix-core path: G = 7 (half-empty last row tile per query page), ragged last half tile of pages
    (Workload("vote_g7", 14, 2, 128, 128, 128 * 3, 128 * (3 + 91), None, "bf16", "f32", 0.0884, extra_phys=2,
              boost_frac=0.1, seed=41), 6),
    (Workload("vote_g2", 4, 2, 128, 128, 128 * 5, 128 * (5 + 200), None, "bf16", "bf16", 0.0884, boost_frac=0.05,
              seed=42), 16),
    # plain kernels: fp32 tensors (means not rounded), and bf16 with a page size without a matrix kernel
    (Workload("vote_f32", 4, 2, 64, 16, 16 * 5, 16 * (5 + 37), None, "f32", "f32", 0.125, boost_frac=0.1, seed=43), 4),
    (Workload("vote_bf16_p64", 8, 2, 128, 64, 64 * 3, 64 * (3 + 50), None, "bf16", "f32", 0.088, boost_frac=0.1,
              seed=44), 5),
]


@pytest.mark.parametrize("w,top_k", VOTE_CASES, ids=lambda v: v.name if isinstance(v, Workload) else str(v))
def test_votes_and_lists(w, top_k):
    *_, differ = vote_parity(w, top_k)
    assert differ == 0, f"{differ} lists differ from the oracle's by near-ties"


@pytest.mark.parametrize("top_k", [0, 1000])
def test_top_k_zero_and_larger_than_the_history(top_k):
    w = VOTE_CASES[0][0]
    *_, sel, cnt, osel, ocnt, differ = vote_parity(w, top_k)
    assert differ == 0


def test_no_history():
    w = VOTE_CASES[1][0].with_(name="vote_nohist", N=128 * 5, boost_frac=0.0)
    x, hx, sel, cnt, osel, ocnt, differ = vote_parity(w, 4)
    assert differ == 0 and (cnt == np.arange(1, w.m + 1)[None, :]).all()


@pytest.mark.parametrize("case", [0, 1])
def test_whole_path_votes_lists_attention(case):
    """Votes -> lists on the GPU, forward and backward over those lists, against the oracle's own
    lists and attention (the lists agree exactly on these seeded inputs)."""
    w, top_k = VOTE_CASES[case]
    x, hx, sel, cnt, osel, ocnt, differ = vote_parity(w, top_k)
    assert differ == 0
    res = gpu_fwd_bwd_qp(w, x, sel, cnt)
    ref = orc.attn_fwd_bwd(pu.shape_of(w), hx["q"], hx["k_pool"], hx["v_pool"], hx["page_table"], hx["d_o"], osel, ocnt,
                           prec="f32")
    gd = w.dtype if w.grad_dtype == "f32" else "bf16"
    pu.check("O", pu.f32(res["o"]), ref["o"], w.dtype)
    pu.check("LSE", pu.f32(res["lse"]), ref["lse"], "bf16")
    pu.check("dQ", pu.f32(res["dq"]), ref["dq"], w.dtype)
    pu.check("dK pool", pu.f32(res["dk_pool"]), ref["dk_pool"], gd)
    pu.check("dV pool", pu.f32(res["dv_pool"]), ref["dv_pool"], gd)


def test_votes_are_deterministic():
    w, top_k = VOTE_CASES[0]
    x = make_inputs(w, "cuda")
    a = gpu_vote(w, x, top_k)
    b = gpu_vote(w, x, top_k)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[2].view(np.uint32), b[2].view(np.uint32))


def _oracle_lists_of_head(w, hx, okb, g0, top_k, taus=None):
    """The oracle's votes and lists of every query page (or of the query pages `taus`) of KV head g0.  vote[g0][tau] depends only on
    the rows of (g0, tau) and on the means of head g0, so each query page is a one-page problem of its
    own; they run side by side in threads (the C function releases the interpreter lock)."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import Shape
    q = hx["q"]
    kb = np.ascontiguousarray(okb[: w.n_past, g0:g0 + 1])
    sub = Shape(w.G, 1, w.D, w.P, w.P, (w.n_past + 1) * w.P, w.sm_scale)

    def one(tau):
        qs = np.ascontiguousarray(q[tau * w.P:(tau + 1) * w.P, g0 * w.G:(g0 + 1) * w.G])
        s, c, v = orc.page_vote_topk(sub, qs, kb, top_k)
        return s[0, 0, : c[0, 0] - 1], v[0, 0]

    taus = list(range(w.m)) if taus is None else list(taus)
    with ThreadPoolExecutor(max_workers=min(16, orc.num_threads())) as ex:
        res = list(ex.map(one, taus))
    sel = np.full((w.m, top_k + w.m), -1, np.int32)
    cnt = np.zeros(w.m, np.int32)
    votes = np.zeros((w.m, w.n_past))
    for tau, (past, v) in zip(taus, res):
        votes[tau] = v
        lst = list(past) + list(range(w.n_past, w.n_past + tau + 1))
        sel[tau, : len(lst)] = lst
        cnt[tau] = len(lst)
    return sel, cnt, votes


def test_votes_path_full_size():
    """1M-token history in the configuration bench.py --retrieval votes times: the votes and lists of
    one KV head against the oracle in full, then sampled rows (O, LSE, dQ) and sampled pages (dK, dV)
    of that head over the oracle's lists, and the identities that hold at any size."""
    import test_gpu_parity_full as full
    w = WORKLOADS["qwen_sparse_1m"]
    top_k, g0 = w.top_k, 1
    x = make_inputs(w, "cuda")
    hx = pu.host_inputs(x)
    sel, cnt, votes, cache = gpu_vote(w, x, top_k)
    sh = pu.shape_of(w)
    okb = orc.page_means(sh, hx["k_pool"], hx["page_table"], 0, w.n_past, np.zeros((w.n, w.Hkv, w.D), np.float32))
    assert np.array_equal(cache[: w.n_past].view(np.uint32), okb[: w.n_past].view(np.uint32)), "page means differ"
    osel_g, ocnt_g, ovotes_g = _oracle_lists_of_head(w, hx, okb, g0, top_k)
    err = np.abs(votes[g0] - ovotes_g) / np.maximum(ovotes_g, 1e-30)
    print(f"votes of head {g0}: max rel {err.max():.2e}", flush=True)
    assert err.max() < VOTE_RTOL
    # lists of the other heads are never read by the oracle calls below (rows and pages of head g0 only)
    osel = np.full((w.Hkv, w.m, top_k + w.m), -1, np.int32)
    ocnt = np.zeros((w.Hkv, w.m), np.int32)
    for g in range(w.Hkv):
        for tau in range(w.m):
            osel[g, tau, : tau + 1] = np.arange(w.n_past, w.n_past + tau + 1)
            ocnt[g, tau] = tau + 1
    osel[g0], ocnt[g0] = osel_g, ocnt_g
    one = w.with_(Hkv=1, Hq=w.G)
    differ = check_lists(one, top_k, sel[g0:g0 + 1], cnt[g0:g0 + 1], osel[g0:g0 + 1], ocnt[g0:g0 + 1], ovotes_g[None])
    assert differ == 0, f"{differ} lists of head {g0} differ from the oracle's by near-ties"
    union = np.unique(osel_g[osel_g >= 0])
    print(f"head {g0}: {len(union)} distinct pages in {w.m} lists of {top_k} + local", flush=True)

    res = gpu_fwd_bwd_qp(w, x, sel, cnt)
    rows = full._sample_rows(w, 200, 3)
    rows = rows[(rows[:, 0] // w.G) == g0]
    assert len(rows) >= 24
    full._check_rows(w, hx, res, osel, ocnt, rows)
    held = np.bincount(osel_g[osel_g >= 0], minlength=w.n)          # lists that hold each page
    pages = [int(union[0]), int(np.argmax(held[: w.n_past])), int(w.n_past), int(w.n_past + w.m // 2), int(w.n - 1)]
    full._check_pages(w, hx, res, osel, ocnt, g0, sorted(set(pages)))
    full._check_identities(w, x, res)
    # pages in no list of head g0 are untouched
    untouched = np.setdiff1d(np.arange(w.n_phys), hx["page_table"][union])
    idx = torch.as_tensor(untouched, device="cuda")
    assert not res["dk_pool"][idx, g0].any() and not res["dv_pool"][idx, g0].any()


def test_votes_path_4m_stress():
    """4M-token history, chunk 8192 (64 query pages), top-k 256, bf16 gradient pool: the largest sizes.
    Votes and lists of three sampled (KV head, query page) pairs against the oracle, rows of those
    query pages over the oracle's lists, and the identities that hold at any size."""
    import test_gpu_parity_full as full
    w = WORKLOADS["qwen_sparse_4m"]
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < 64 * 2 ** 30:
        pytest.skip("needs about 64 GiB of free device memory")
    top_k, g0 = w.top_k, 2
    taus = [0, 37, w.m - 1]
    x = make_inputs(w, "cuda")
    hx = pu.host_inputs(x)
    sel, cnt, votes, cache = gpu_vote(w, x, top_k)
    sh = pu.shape_of(w)
    okb = orc.page_means(sh, hx["k_pool"], hx["page_table"], 0, w.n_past, np.zeros((w.n, w.Hkv, w.D), np.float32))
    assert np.array_equal(cache[: w.n_past].view(np.uint32), okb[: w.n_past].view(np.uint32)), "page means differ"
    osel_g, ocnt_g, ovotes_g = _oracle_lists_of_head(w, hx, okb, g0, top_k, taus)
    for tau in taus:
        err = np.abs(votes[g0, tau] - ovotes_g[tau]) / np.maximum(ovotes_g[tau], 1e-30)
        assert err.max() < VOTE_RTOL, (tau, err.max())
        assert cnt[g0, tau] == ocnt_g[tau]
        if not np.array_equal(sel[g0, tau], osel_g[tau]):   # accepted only as a tie within the tolerance
            v = ovotes_g[tau]
            vk = np.sort(v)[::-1][top_k - 1]
            past = sel[g0, tau, :top_k]
            assert v[past].min() >= vk * (1 - VOTE_RTOL)
            assert np.delete(v, past).max() <= vk * (1 + VOTE_RTOL)
            pytest.fail(f"list of query page {tau} differs from the oracle's by a near-tie")
    assert (np.diff(sel[:, :, :top_k], axis=2) > 0).all()
    assert (cnt == top_k + 1 + np.arange(w.m)[None, :]).all()

    res = gpu_fwd_bwd_qp(w, x, sel, cnt)
    osel = np.full((w.Hkv, w.m, top_k + w.m), -1, np.int32)
    ocnt = np.zeros((w.Hkv, w.m), np.int32)
    for tau in taus:
        osel[g0, tau], ocnt[g0, tau] = osel_g[tau], ocnt_g[tau]
    rng = np.random.default_rng(4)
    rows = np.array([(g0 * w.G + int(rng.integers(w.G)), tau * w.P + int(i)) for tau in taus
                     for i in (0, 31, 32, w.P - 1, int(rng.integers(w.P)), int(rng.integers(w.P)))], dtype=np.int32)
    full._check_rows(w, hx, res, osel, ocnt, rows)
    full._check_identities(w, x, res)


def test_benchmark_sequence_of_16_chunks_with_votes():
    """The sequence bench.py --retrieval votes --cached-means times: 16 calls with the history growing by one
    chunk per call, page means cached once, workspaces and outputs allocated for the longest history, gradient
    pools persisting.  Checked: lists of two query pages of one KV head in the last call against the oracle,
    rows of those query pages, and the pools after all 16 calls through <dV, V> = sum over calls <dO, O> and
    <dK, K> = sum <dQ, Q>; pages in no list of any call are untouched."""
    import test_gpu_parity_full as full
    w = WORKLOADS["qwen_sparse_1m"]
    top_k, g0, taus = w.top_k, 3, [5, w.m - 1]
    x = make_inputs(w, "cuda")
    hx = pu.host_inputs(x)
    dev = x["q"].device
    steps = w.extra_phys // w.m + 1
    gdt = torch_dtype(w.grad_dtype)
    descs = [api.make_desc(x["q"], x["k_pool"], w.N + s * w.C, w.sm_scale, gdt) for s in range(steps)]
    ws = {op: torch.empty(api.workspace_bytes(descs[-1], top_k, op), dtype=torch.uint8, device=dev)
          for op in (api.OP_VOTE_TOPK, api.OP_ATTN_FWD_QP, api.OP_ATTN_BWD_QP)}
    sel = torch.empty((w.Hkv, w.m, top_k + w.m), dtype=torch.int32, device=dev)
    cnt = torch.empty((w.Hkv, w.m), dtype=torch.int32, device=dev)
    votes = torch.zeros((w.Hkv, w.m, w.n_phys - w.m), dtype=torch.float32, device=dev)
    o = torch.empty_like(x["q"])
    lse = torch.empty((w.Hq, w.C), dtype=torch.float32, device=dev)
    dq = torch.empty_like(x["q"])
    cache = torch.zeros((w.n_phys, w.Hkv, w.D), dtype=torch.float32, device=dev)
    api.page_means(descs[-1], x["k_pool"], x["page_table"], 0, w.n_phys, cache)
    acc = torch.zeros((4, w.Hkv), dtype=torch.float64, device=dev)   # rhs_v, rhs_k, mass_v, mass_k
    touched = [set() for _ in range(w.Hkv)]
    for s, desc in enumerate(descs):
        last = s == steps - 1
        api.page_vote_topk(desc, x["q"], cache, top_k, sel, cnt, votes_out=votes if last else None,
                           workspace=ws[api.OP_VOTE_TOPK])
        api.paged_attn_fwd_qp(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], sel, cnt, o, lse,
                              ws[api.OP_ATTN_FWD_QP])
        api.paged_attn_bwd_qp(desc, x["q"], x["k_pool"], x["v_pool"], x["page_table"], o, lse, x["d_o"], x["dk_pool"],
                              x["dv_pool"], sel, cnt, dq, ws[api.OP_ATTN_BWD_QP])
        for g in range(w.Hkv):
            hs = slice(g * w.G, (g + 1) * w.G)
            acc[0, g] += (x["d_o"][:, hs].double() * o[:, hs].double()).sum()
            acc[1, g] += (dq[:, hs].double() * x["q"][:, hs].double()).sum()
            acc[2, g] += (x["d_o"][:, hs].double().abs() * o[:, hs].double().abs()).sum()
            acc[3, g] += (dq[:, hs].double().abs() * x["q"][:, hs].double().abs()).sum()
        hsel = sel.cpu().numpy()
        for g in range(w.Hkv):
            touched[g] |= set(hsel[g][hsel[g] >= 0].tolist())
    torch.cuda.synchronize()
    hcnt = cnt.cpu().numpy()

    # the last call: two query pages of head g0 against the oracle
    lw = w.with_(name="qwen_sparse_1m_last", N=w.N + (steps - 1) * w.C, extra_phys=0)
    okb = orc.page_means(pu.shape_of(lw), hx["k_pool"], hx["page_table"], 0, lw.n_past,
                         np.zeros((lw.n, lw.Hkv, lw.D), np.float32))
    assert np.array_equal(cache[: lw.n_past].cpu().numpy().view(np.uint32), okb[: lw.n_past].view(np.uint32))
    osel_g, ocnt_g, ovotes_g = _oracle_lists_of_head(lw, hx, okb, g0, top_k, taus)
    hv = votes[g0, :, : lw.n_past].cpu().numpy()
    osel = np.full((lw.Hkv, lw.m, top_k + lw.m), -1, np.int32)
    ocnt = np.zeros((lw.Hkv, lw.m), np.int32)
    for tau in taus:
        err = np.abs(hv[tau] - ovotes_g[tau]) / np.maximum(ovotes_g[tau], 1e-30)
        assert err.max() < VOTE_RTOL, (tau, err.max())
        assert hcnt[g0, tau] == ocnt_g[tau]
        assert np.array_equal(hsel[g0, tau], osel_g[tau]), f"list of query page {tau} differs from the oracle's"
        osel[g0, tau], ocnt[g0, tau] = osel_g[tau], ocnt_g[tau]
    rng = np.random.default_rng(6)
    rows = np.array([(g0 * w.G + int(rng.integers(w.G)), tau * w.P + int(i)) for tau in taus
                     for i in (0, 31, 32, w.P - 1, int(rng.integers(w.P)), int(rng.integers(w.P)))], dtype=np.int32)
    full._check_rows(lw, hx, dict(o=o, lse=lse, dq=dq), osel, ocnt, rows)

    # the pools after the 16 calls
    acc = acc.cpu().numpy()
    for g in range(w.Hkv):
        lhs_v = (x["dv_pool"][:, g].double() * x["v_pool"][:, g].double()).sum().item()
        lhs_k = (x["dk_pool"][:, g].double() * x["k_pool"][:, g].double()).sum().item()
        assert abs(lhs_v - acc[0, g]) <= 5e-3 * acc[2, g], (g, lhs_v, acc[0, g])
        assert abs(lhs_k - acc[1, g]) <= 5e-3 * acc[3, g], (g, lhs_k, acc[1, g])
        untouched = np.setdiff1d(np.arange(w.n_phys), hx["page_table"][np.array(sorted(touched[g]))])
        idx = torch.as_tensor(untouched, device=dev)
        assert not x["dk_pool"][idx, g].any() and not x["dv_pool"][idx, g].any()
