"""Pins of the oracle's offload steps (paper Sec. 4.3: the KV cache and its gradients live in host memory,
the pages a chunk attends are fetched, their gradients written back).  They are data movement, so the
pins are structural: what moves where, what is left alone, and that attention over the staged pages is
the attention over the resident pool, bit for bit."""
import numpy as np

import oracle
from oracle import Shape


def _problem(seed, Hq=4, Hkv=2, D=16, P=8, C=24, N=120, k_sel=3, extra=3):
    rng = np.random.default_rng(seed)
    sh = Shape(Hq, Hkv, D, P, C, N, 0.25)
    n_phys = sh.n + extra
    pt = rng.permutation(n_phys)[: sh.n].astype(np.int32)
    k = rng.standard_normal((n_phys, Hkv, P, D)).astype(np.float32)
    v = rng.standard_normal((n_phys, Hkv, P, D)).astype(np.float32)
    q = rng.standard_normal((C, Hq, D)).astype(np.float32)
    d_o = rng.standard_normal((C, Hq, D)).astype(np.float32)
    sel = np.full((Hkv, k_sel + sh.m), -1, np.int32)
    for g in range(Hkv):
        sel[g] = np.concatenate([np.sort(rng.choice(sh.n_past, k_sel, replace=False)), np.arange(sh.n_past, sh.n)])
    cnt = np.full(Hkv, k_sel + sh.m, np.int32)
    return rng, sh, pt, k, v, q, d_o, sel, cnt


def test_plan_numbers_the_union_of_the_lists_in_page_order():
    _, sh, pt, k, v, q, d_o, sel, cnt = _problem(1)
    table, slots, mask = oracle.offload_plan(sh, sel, cnt)
    union = sorted(set(sel[0, : cnt[0]]) | set(sel[1, : cnt[1]]))
    assert list(slots) == union
    for l in range(sh.n):
        assert table[l] == (union.index(l) if l in union else -1)
        assert mask[l] == (1 if l in sel[0, : cnt[0]] else 0) + (2 if l in sel[1, : cnt[1]] else 0)
    # entries beyond sel_count are not read
    sel2 = sel.copy()
    cnt2 = cnt.copy()
    cnt2[1] -= 1
    sel2[1, cnt2[1]] = 0
    t2, s2, _ = oracle.offload_plan(sh, sel2, cnt2)
    assert list(s2) == sorted(set(sel[0, : cnt[0]]) | set(sel[1, : cnt2[1]]))


def test_plan_over_per_query_page_lists_is_the_plan_over_their_union():
    rng, sh, pt, k, v, q, d_o, sel, cnt = _problem(5)
    sel3 = np.full((sh.Hkv, sh.m, 2 + sh.m), -1, np.int32)
    cnt3 = np.zeros((sh.Hkv, sh.m), np.int32)
    for g in range(sh.Hkv):
        for tau in range(sh.m):
            lst = sorted(rng.choice(sh.n_past, 2, replace=False)) + list(range(sh.n_past, sh.n_past + tau + 1))
            sel3[g, tau, : len(lst)] = lst
            cnt3[g, tau] = len(lst)
    table, slots, mask = oracle.offload_plan(sh, sel3, cnt3)
    per_head = [set(int(l) for tau in range(sh.m) for l in sel3[g, tau, : cnt3[g, tau]]) for g in range(sh.Hkv)]
    assert list(slots) == sorted(per_head[0] | per_head[1])
    for l in range(sh.n):
        assert mask[l] == sum(1 << g for g in range(sh.Hkv) if l in per_head[g])


def test_fetch_moves_exactly_the_listed_head_page_tiles():
    rng, sh, pt, k, v, q, d_o, sel, cnt = _problem(2)
    table, slots, mask = oracle.offload_plan(sh, sel, cnt)
    junk_k = rng.standard_normal((len(slots), sh.Hkv, sh.P, sh.D)).astype(np.float32)
    junk_v = rng.standard_normal(junk_k.shape).astype(np.float32)
    sk, sv = oracle.offload_fetch(sh, k, v, pt, slots, mask, junk_k, junk_v)
    for s, l in enumerate(slots):
        for g in range(sh.Hkv):
            if l in sel[g, : cnt[g]]:
                assert np.array_equal(sk[s, g], k[pt[l], g]) and np.array_equal(sv[s, g], v[pt[l], g])
            else:   # a page another head listed: this head's tile of the slot is left alone
                assert np.array_equal(sk[s, g], junk_k[s, g]) and np.array_equal(sv[s, g], junk_v[s, g])


def test_writeback_adds_the_listed_tiles_and_nothing_else():
    rng, sh, pt, k, v, q, d_o, sel, cnt = _problem(3)
    table, slots, mask = oracle.offload_plan(sh, sel, cnt)
    sdk = rng.standard_normal((len(slots), sh.Hkv, sh.P, sh.D)).astype(np.float32)
    sdv = rng.standard_normal(sdk.shape).astype(np.float32)
    hk0 = rng.standard_normal(k.shape).astype(np.float32)
    hv0 = rng.standard_normal(k.shape).astype(np.float32)
    hk, hv = oracle.offload_writeback(sh, sdk, sdv, hk0, hv0, pt, slots, mask)
    touched = np.zeros(k.shape[:2], bool)
    for g in range(sh.Hkv):
        for l in sel[g, : cnt[g]]:
            touched[pt[l], g] = True
            assert np.array_equal(hk[pt[l], g], hk0[pt[l], g] + sdk[table[l], g])
            assert np.array_equal(hv[pt[l], g], hv0[pt[l], g] + sdv[table[l], g])
    assert np.array_equal(hk[~touched], hk0[~touched]) and np.array_equal(hv[~touched], hv0[~touched])


def test_attention_over_the_staged_pages_is_the_attention_over_the_resident_pool():
    rng, sh, pt, k, v, q, d_o, sel, cnt = _problem(4)
    ref = oracle.attn_fwd_bwd(sh, q, k, v, pt, d_o, sel, cnt, prec="f32")
    table, slots, mask = oracle.offload_plan(sh, sel, cnt)
    shape = (len(slots), sh.Hkv, sh.P, sh.D)
    nan = np.full(shape, np.nan, np.float32)       # tiles that are never fetched must never be read
    sk, sv = oracle.offload_fetch(sh, k, v, pt, slots, mask, nan, nan)
    staged_pt = np.where(table >= 0, table, 0).astype(np.int32)
    got = oracle.attn_fwd_bwd(sh, q, sk, sv, staged_pt, d_o, sel, cnt, prec="f32")
    for key in ("o", "lse", "dq"):
        assert np.array_equal(got[key], ref[key]), key
    hk, hv = oracle.offload_writeback(sh, got["dk_pool"], got["dv_pool"], np.zeros_like(k), np.zeros_like(k), pt, slots,
                                      mask)
    assert np.array_equal(hk, ref["dk_pool"]) and np.array_equal(hv, ref["dv_pool"])


def test_staged_attention_with_per_query_page_lists():
    rng, sh, pt, k, v, q, d_o, sel, cnt = _problem(6)
    sel3 = np.full((sh.Hkv, sh.m, 2 + sh.m), -1, np.int32)
    cnt3 = np.zeros((sh.Hkv, sh.m), np.int32)
    for g in range(sh.Hkv):
        for tau in range(sh.m):
            lst = sorted(rng.choice(sh.n_past, 2, replace=False)) + list(range(sh.n_past, sh.n_past + tau + 1))
            sel3[g, tau, : len(lst)] = lst
            cnt3[g, tau] = len(lst)
    ref = oracle.attn_fwd_bwd(sh, q, k, v, pt, d_o, sel3, cnt3, prec="f32")
    table, slots, mask = oracle.offload_plan(sh, sel3, cnt3)
    nan = np.full((len(slots), sh.Hkv, sh.P, sh.D), np.nan, np.float32)
    sk, sv = oracle.offload_fetch(sh, k, v, pt, slots, mask, nan, nan)
    got = oracle.attn_fwd_bwd(sh, q, sk, sv, np.where(table >= 0, table, 0).astype(np.int32), d_o, sel3, cnt3, prec="f32")
    for key in ("o", "lse", "dq"):
        assert np.array_equal(got[key], ref[key]), key
    hk, hv = oracle.offload_writeback(sh, got["dk_pool"], got["dv_pool"], np.zeros_like(k), np.zeros_like(k), pt, slots, mask)
    assert np.array_equal(hk, ref["dk_pool"]) and np.array_equal(hv, ref["dv_pool"])
