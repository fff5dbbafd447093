"""Pins of the oracle's retrieval by voting (paper Sec. 4.2, the scoring equation: per query token a
softmax over the key pages, summed over the tokens of a query page, top-K per query page) and of the
attention with one page list per query page.  Checked against things other than the oracle: a
library routine (torch SDPA with the page means as keys and the identity as values returns the
per-token distributions; SDPA + autograd with an explicit mask for the attention), closed forms
(zero queries, the hard-max limit), invariants (every token-head spreads exactly one vote), and
brute-force sorting."""
import math

import numpy as np
import pytest
import torch

import oracle
from oracle import Shape


def _problem(seed, Hq=4, Hkv=2, D=16, P=4, C=12, N=52, extra_phys=2, scale=None):
    rng = np.random.default_rng(seed)
    sh = Shape(Hq, Hkv, D, P, C, N, (1.0 / math.sqrt(D)) if scale is None else scale)
    n_phys = sh.n + extra_phys
    pt = rng.permutation(n_phys)[: sh.n].astype(np.int32)
    k = rng.standard_normal((n_phys, Hkv, P, D))
    v = rng.standard_normal((n_phys, Hkv, P, D))
    q = rng.standard_normal((C, Hq, D))
    return rng, sh, pt, k, v, q


def _means(sh, k, pt):
    return oracle.page_means(sh, k, pt, 0, sh.n, np.zeros((sh.n, sh.Hkv, sh.D), np.float32))


def _votes_by_sdpa(sh, q, kbar):
    """Library special case: attention over the page means with identity values returns each
    token's distribution over the pages; sum over the tokens of a query page and the heads of a group."""
    qh = torch.tensor(q, dtype=torch.float64).permute(1, 0, 2)                         # [Hq][C][D]
    kh = torch.tensor(kbar[: sh.n_past], dtype=torch.float64).permute(1, 0, 2)          # [Hkv][n_past][D]
    kh = kh.repeat_interleave(sh.G, dim=0)
    eye = torch.eye(sh.n_past, dtype=torch.float64).expand(sh.Hq, -1, -1)
    p = torch.nn.functional.scaled_dot_product_attention(qh, kh, eye, scale=sh.sm_scale)  # [Hq][C][n_past]
    p = p.reshape(sh.Hkv, sh.G, sh.m, sh.P, sh.n_past)
    return p.sum(dim=(1, 3)).numpy()                                                   # [Hkv][m][n_past]


def _expected_lists(sh, votes, top_k):
    """Full sort by (vote descending, id ascending), then the visible local pages, ascending."""
    k_eff = min(top_k, sh.n_past)
    sel = np.full((sh.Hkv, sh.m, top_k + sh.m), -1, np.int32)
    cnt = np.zeros((sh.Hkv, sh.m), np.int32)
    for g in range(sh.Hkv):
        for tau in range(sh.m):
            order = sorted(range(sh.n_past), key=lambda l: (-votes[g, tau, l], l))[:k_eff]
            lst = sorted(order) + list(range(sh.n_past, sh.n_past + tau + 1))
            sel[g, tau, : len(lst)] = lst
            cnt[g, tau] = len(lst)
    return sel, cnt


@pytest.mark.parametrize("seed", [1, 2])
def test_votes_equal_library_attention_over_the_page_means(seed):
    _, sh, pt, k, _, q = _problem(seed)
    kbar = _means(sh, k, pt)
    _, _, votes = oracle.page_vote_topk(sh, q, kbar, 3)
    want = _votes_by_sdpa(sh, q, kbar)
    assert np.allclose(votes, want, rtol=1e-12, atol=1e-14)


def test_every_token_head_spreads_exactly_one_vote():
    _, sh, pt, k, _, q = _problem(3, Hq=6, Hkv=2, P=8, C=24, N=120)
    _, _, votes = oracle.page_vote_topk(sh, q, _means(sh, k, pt), 4)
    assert np.allclose(votes.sum(axis=2), sh.P * sh.G, rtol=1e-12)
    assert (votes > 0).all()


@pytest.mark.parametrize("top_k", [0, 1, 3, 100])
def test_lists_against_brute_force_sort(top_k):
    _, sh, pt, k, _, q = _problem(4)
    sel, cnt, votes = oracle.page_vote_topk(sh, q, _means(sh, k, pt), top_k)
    wsel, wcnt = _expected_lists(sh, votes, top_k)
    assert np.array_equal(sel, wsel) and np.array_equal(cnt, wcnt)
    # structure: ascending, kept votes >= dropped votes, exactly the visible local pages at the end
    for g in range(sh.Hkv):
        for tau in range(sh.m):
            lst = sel[g, tau, : cnt[g, tau]]
            assert (np.diff(lst) > 0).all()
            past = lst[lst < sh.n_past]
            assert list(lst[len(past):]) == list(range(sh.n_past, sh.n_past + tau + 1))
            dropped = np.setdiff1d(np.arange(sh.n_past), past)
            if len(past) and len(dropped):
                assert votes[g, tau, past].min() >= votes[g, tau, dropped].max()


def test_zero_queries_give_uniform_votes_and_the_lowest_ids():
    _, sh, pt, k, _, q = _problem(5)
    sel, cnt, votes = oracle.page_vote_topk(sh, np.zeros_like(q), _means(sh, k, pt), 3)
    assert np.allclose(votes, sh.P * sh.G / sh.n_past, rtol=1e-13)
    for g in range(sh.Hkv):
        for tau in range(sh.m):
            assert list(sel[g, tau, :3]) == [0, 1, 2]   # exact ties go to the lower logical id


def test_hard_max_limit_counts_each_tokens_best_page():
    # a very large scale turns every token's distribution into a one-hot on its best page: the votes
    # become the histogram of arg-max pages, which pins the axis of the softmax (over key pages)
    _, sh, pt, k, _, q = _problem(6, scale=1e6)
    kbar = _means(sh, k, pt)
    _, _, votes = oracle.page_vote_topk(sh, q, kbar, 2)
    for g in range(sh.Hkv):
        for tau in range(sh.m):
            hist = np.zeros(sh.n_past)
            for h in range(g * sh.G, (g + 1) * sh.G):
                for i in range(tau * sh.P, (tau + 1) * sh.P):
                    dots = kbar[: sh.n_past, g].astype(np.float64) @ q[i, h]
                    hist[int(np.argmax(dots))] += 1
            assert np.allclose(votes[g, tau], hist, atol=1e-6)


def test_identical_tokens_rank_pages_like_the_plain_dot_product():
    rng, sh, pt, k, _, q = _problem(7, Hq=2, Hkv=2)   # G = 1
    tok = rng.standard_normal((sh.Hq, sh.D))
    qq = np.broadcast_to(tok, (sh.C, sh.Hq, sh.D)).copy()
    kbar = _means(sh, k, pt)
    sel, cnt, votes = oracle.page_vote_topk(sh, qq, kbar, 4)
    for g in range(sh.Hkv):
        dots = kbar[: sh.n_past, g].astype(np.float64) @ tok[g]
        want = np.sort(np.argsort(-dots, kind="stable")[:4])
        for tau in range(sh.m):
            assert list(sel[g, tau, :4]) == list(want)


def test_scale_enters_before_the_softmax():
    _, sh, pt, k, _, q = _problem(8)
    kbar = _means(sh, k, pt)
    _, _, v1 = oracle.page_vote_topk(sh, q, kbar, 2)
    sh2 = Shape(sh.Hq, sh.Hkv, sh.D, sh.P, sh.C, sh.N, 2 * sh.sm_scale)
    _, _, v2 = oracle.page_vote_topk(sh2, 0.5 * q, kbar, 2)
    assert np.allclose(v1, v2, rtol=1e-12)
    _, _, v3 = oracle.page_vote_topk(sh2, q, kbar, 2)
    assert not np.allclose(v1, v3, rtol=1e-3)


def test_vote_placement_invariance_and_cache_only():
    rng, sh, pt, k, _, q = _problem(9)
    kbar = _means(sh, k, pt)
    sel, cnt, votes = oracle.page_vote_topk(sh, q, kbar, 3)
    perm = rng.permutation(k.shape[0])
    inv = np.argsort(perm)
    kbar2 = _means(sh, k[perm], inv[pt].astype(np.int32))
    sel2, cnt2, votes2 = oracle.page_vote_topk(sh, q, kbar2, 3)
    assert np.array_equal(sel, sel2) and np.array_equal(cnt, cnt2) and np.array_equal(votes, votes2)
    # rows of the cache at and beyond n_past (the chunk's own pages) are never candidates
    kbar3 = kbar.copy()
    kbar3[sh.n_past:] = 1e6
    sel3, _, votes3 = oracle.page_vote_topk(sh, q, kbar3, 3)
    assert np.array_equal(sel, sel3) and np.array_equal(votes, votes3)


def test_bf16_queries_round_the_means_to_bf16_first():
    _, sh, pt, k, _, q = _problem(10)
    qb = (q.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    q_as_f = (qb.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    kbar = _means(sh, k, pt)
    # independent rounding to bf16 (nearest even) through torch
    kbar_r = torch.tensor(kbar).to(torch.bfloat16).to(torch.float32).numpy()
    _, _, v_bf = oracle.page_vote_topk(sh, qb, kbar, 3)
    _, _, v_ref = oracle.page_vote_topk(sh, q_as_f, kbar_r, 3, kbar_round_bf16=False)
    assert np.array_equal(v_bf, v_ref)
    _, _, v_unrounded = oracle.page_vote_topk(sh, q_as_f, kbar, 3, kbar_round_bf16=False)
    assert not np.array_equal(v_bf, v_unrounded)


def test_no_history_gives_only_local_pages():
    _, sh, pt, k, _, q = _problem(11, C=12, N=12)
    sel, cnt, votes = oracle.page_vote_topk(sh, q, np.zeros((sh.n, sh.Hkv, sh.D), np.float32), 3)
    assert votes.shape[2] == 0
    for g in range(sh.Hkv):
        for tau in range(sh.m):
            assert cnt[g, tau] == tau + 1 and list(sel[g, tau, : tau + 1]) == list(range(tau + 1))


# ---- attention with one list per query page -------------------------------------------------------

def _flatten(sh, pool, pt):
    return pool[pt[: sh.n]].transpose(0, 2, 1, 3).reshape(sh.N, sh.Hkv, sh.D)


def _mask_qp(sh, sel, cnt):
    """[Hkv][C][N] visibility from the definition: t <= a_i and page of t in the list of (g, i / P)."""
    msk = np.zeros((sh.Hkv, sh.C, sh.N), dtype=bool)
    t = np.arange(sh.N)
    for g in range(sh.Hkv):
        for i in range(sh.C):
            pages = sel[g, i // sh.P, : cnt[g, i // sh.P]]
            msk[g, i] = (t <= sh.N - sh.C + i) & np.isin(t // sh.P, pages)
    return msk


def _torch_reference(sh, q, d_o, k, v, pt, msk):
    kf = torch.tensor(_flatten(sh, k, pt), dtype=torch.float64, requires_grad=True)
    vf = torch.tensor(_flatten(sh, v, pt), dtype=torch.float64, requires_grad=True)
    qt = torch.tensor(q, dtype=torch.float64, requires_grad=True)
    msk_h = torch.tensor(msk).repeat_interleave(sh.G, dim=0)
    qh = qt.permute(1, 0, 2)
    kh = kf.permute(1, 0, 2).repeat_interleave(sh.G, dim=0)
    vh = vf.permute(1, 0, 2).repeat_interleave(sh.G, dim=0)
    o = torch.nn.functional.scaled_dot_product_attention(qh, kh, vh, attn_mask=msk_h, scale=sh.sm_scale)
    logits = (qh @ kh.transpose(1, 2)) * sh.sm_scale
    lse = torch.logsumexp(logits.masked_fill(~msk_h, -math.inf), dim=-1)
    o.backward(torch.tensor(d_o, dtype=torch.float64).permute(1, 0, 2))
    return (o.permute(1, 0, 2).detach().numpy(), lse.detach().numpy(), qt.grad.numpy(), kf.grad.numpy(),
            vf.grad.numpy())


def _rand_lists(sh, k_sel, rng):
    sel = np.full((sh.Hkv, sh.m, k_sel + sh.m), -1, np.int32)
    cnt = np.zeros((sh.Hkv, sh.m), np.int32)
    for g in range(sh.Hkv):
        for tau in range(sh.m):
            past = np.sort(rng.choice(sh.n_past, size=k_sel, replace=False))
            lst = list(past) + list(range(sh.n_past, sh.n_past + tau + 1))
            sel[g, tau, : len(lst)] = lst
            cnt[g, tau] = len(lst)
    return sel, cnt


@pytest.mark.parametrize("prec,tol", [("f64", 1e-10), ("f32", 2e-5)])
def test_attention_with_per_query_page_lists_against_library_sdpa_autograd(prec, tol):
    rng, sh, pt, k, v, q = _problem(21, Hq=6, Hkv=2, D=16, P=8, C=32, N=128)
    d_o = rng.standard_normal(q.shape)
    sel, cnt = _rand_lists(sh, 4, rng)
    res = oracle.attn_fwd_bwd(sh, q, k, v, pt, d_o, sel, cnt, prec=prec)
    o, lse, dq, dkf, dvf = _torch_reference(sh, q, d_o, k, v, pt, _mask_qp(sh, sel, cnt))

    def rel(a, b):
        return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30)

    assert rel(res["o"], o) < tol and rel(res["lse"], lse) < tol and rel(res["dq"], dq) < tol
    assert rel(_flatten(sh, res["dk_pool"], pt), dkf) < tol
    assert rel(_flatten(sh, res["dv_pool"], pt), dvf) < tol
    # pages in no list stay untouched
    for g in range(sh.Hkv):
        used = np.unique(sel[g][sel[g] >= 0])
        unused = np.setdiff1d(np.arange(sh.n), used)
        assert not res["dk_pool"][pt[unused], g].any() and not res["dv_pool"][pt[unused], g].any()


def test_equal_lists_for_every_query_page_reduce_to_one_list_per_head():
    rng, sh, pt, k, v, q = _problem(22, Hq=4, Hkv=2, D=16, P=8, C=24, N=96)
    d_o = rng.standard_normal(q.shape)
    past = [np.sort(rng.choice(sh.n_past, size=3, replace=False)) for _ in range(sh.Hkv)]
    sel1 = np.stack([np.concatenate([past[g], np.arange(sh.n_past, sh.n)]) for g in range(sh.Hkv)]).astype(np.int32)
    cnt1 = np.full(sh.Hkv, 3 + sh.m, np.int32)
    sel3 = np.full((sh.Hkv, sh.m, 3 + sh.m), -1, np.int32)
    cnt3 = np.zeros((sh.Hkv, sh.m), np.int32)
    for g in range(sh.Hkv):
        for tau in range(sh.m):
            lst = list(past[g]) + list(range(sh.n_past, sh.n_past + tau + 1))
            sel3[g, tau, : len(lst)] = lst
            cnt3[g, tau] = len(lst)
    a = oracle.attn_fwd_bwd(sh, q, k, v, pt, d_o, sel1, cnt1, prec="f64")
    b = oracle.attn_fwd_bwd(sh, q, k, v, pt, d_o, sel3, cnt3, prec="f64")
    for key in ("o", "lse", "dq", "dk_pool", "dv_pool"):
        assert np.array_equal(a[key], b[key]), key


def test_row_subset_and_unit_subset_with_per_query_page_lists():
    rng, sh, pt, k, v, q = _problem(23, Hq=4, Hkv=2, D=16, P=8, C=24, N=96)
    d_o = rng.standard_normal(q.shape)
    sel, cnt = _rand_lists(sh, 3, rng)
    full = oracle.attn_fwd_bwd(sh, q, k, v, pt, d_o, sel, cnt, prec="f64")
    rows = np.array([[0, 0], [3, 23], [2, 9], [1, 16]], np.int32)
    o, lse = oracle.attn_fwd(sh, q, k, v, pt, sel, cnt, rows=rows, prec="f64")
    dq = oracle.attn_bwd_dq(sh, q, k, v, pt, full["lse"], full["delta"], d_o, sel, cnt, rows=rows, prec="f64")
    for r, (h, i) in enumerate(rows):
        assert np.array_equal(o[r], full["o"][i, h]) and lse[r] == full["lse"][h, i]
        assert np.array_equal(dq[r], full["dq"][i, h])
    g, l = 1, int(sel[1, 2, 0])
    dk = np.zeros_like(full["dk_pool"])
    dv = np.zeros_like(full["dv_pool"])
    oracle.attn_bwd_dkv(sh, q, k, v, pt, full["lse"], full["delta"], d_o, dk, dv, sel, cnt,
                        units=np.array([[g, l]], np.int32), prec="f64")
    assert np.array_equal(dk[pt[l], g], full["dk_pool"][pt[l], g])
    assert np.array_equal(dv[pt[l], g], full["dv_pool"][pt[l], g])
    dk[pt[l], g] = 0
    dv[pt[l], g] = 0
    assert not dk.any() and not dv.any()
