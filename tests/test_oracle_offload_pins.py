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


def _qp_lists(rng, sh):
    sel3 = np.full((sh.Hkv, sh.m, 2 + sh.m), -1, np.int32)
    cnt3 = np.zeros((sh.Hkv, sh.m), np.int32)
    for g in range(sh.Hkv):
        for tau in range(sh.m):
            lst = sorted(rng.choice(sh.n_past, 2, replace=False)) + list(range(sh.n_past, sh.n_past + tau + 1))
            sel3[g, tau, : len(lst)] = lst
            cnt3[g, tau] = len(lst)
    return sel3, cnt3


def test_stage_table_numbers_the_union_of_the_lists_in_page_order():
    _, sh, pt, k, v, q, d_o, sel, cnt = _problem(1)
    table, n_union = oracle.offload_stage_table(sh, sel, cnt)
    union = sorted(set(sel[0, : cnt[0]]) | set(sel[1, : cnt[1]]))
    assert n_union == len(union)
    for l in range(sh.n):
        assert table[l] == (union.index(l) if l in union else -1)
    # entries beyond sel_count are not read
    sel2 = sel.copy()
    cnt2 = cnt.copy()
    cnt2[1] -= 1
    sel2[1, cnt2[1]] = 0
    t2, n2 = oracle.offload_stage_table(sh, sel2, cnt2)
    union2 = sorted(set(sel[0, : cnt[0]]) | set(sel[1, : cnt2[1]]))
    assert n2 == len(union2) and [l for l in range(sh.n) if t2[l] >= 0] == union2


def test_stage_table_over_per_query_page_lists_is_the_table_over_their_union():
    rng, sh, pt, k, v, q, d_o, sel, cnt = _problem(5)
    sel3, cnt3 = _qp_lists(rng, sh)
    table, n_union = oracle.offload_stage_table(sh, sel3, cnt3)
    per_head = [set(int(l) for tau in range(sh.m) for l in sel3[g, tau, : cnt3[g, tau]]) for g in range(sh.Hkv)]
    union = sorted(per_head[0] | per_head[1])
    assert n_union == len(union) and [l for l in range(sh.n) if table[l] >= 0] == union
    assert [int(table[l]) for l in union] == list(range(len(union)))


def test_stage_table_never_points_outside_a_staging_pool_that_is_too_small():
    _, sh, pt, k, v, q, d_o, sel, cnt = _problem(7)
    full, n_union = oracle.offload_stage_table(sh, sel, cnt)
    cap = n_union - 2
    table, n2 = oracle.offload_stage_table(sh, sel, cnt, capacity=cap)
    assert n2 == n_union > cap                      # the caller can see that the pools were too small
    assert table.max() < cap
    for l in range(sh.n):
        assert table[l] == (full[l] if full[l] < cap else 0)
    # the tiles of the overflowing pages do not move
    rng = np.random.default_rng(0)
    junk = rng.standard_normal((cap, sh.Hkv, sh.P, sh.D)).astype(np.float32)
    sk, sv = oracle.offload_fetch(sh, k, v, pt, sel, cnt, junk, junk)
    for g in range(sh.Hkv):
        for l in sel[g, : cnt[g]]:
            if full[l] < cap:
                assert np.array_equal(sk[full[l], g], k[pt[l], g])
    moved = {(int(full[l]), g) for g in range(sh.Hkv) for l in sel[g, : cnt[g]] if full[l] < cap}
    for s_ in range(cap):
        for g in range(sh.Hkv):
            if (s_, g) not in moved:
                assert np.array_equal(sk[s_, g], junk[s_, g])


def test_fetch_moves_exactly_the_listed_head_page_tiles():
    rng, sh, pt, k, v, q, d_o, sel, cnt = _problem(2)
    table, n_union = oracle.offload_stage_table(sh, sel, cnt)
    junk_k = rng.standard_normal((n_union, sh.Hkv, sh.P, sh.D)).astype(np.float32)
    junk_v = rng.standard_normal(junk_k.shape).astype(np.float32)
    sk, sv = oracle.offload_fetch(sh, k, v, pt, sel, cnt, junk_k, junk_v)
    slots = [l for l in range(sh.n) if table[l] >= 0]
    for s, l in enumerate(slots):
        for g in range(sh.Hkv):
            if l in sel[g, : cnt[g]]:
                assert np.array_equal(sk[s, g], k[pt[l], g]) and np.array_equal(sv[s, g], v[pt[l], g])
            else:   # a page another head listed: this head's tile of the slot is left alone
                assert np.array_equal(sk[s, g], junk_k[s, g]) and np.array_equal(sv[s, g], junk_v[s, g])


def test_writeback_adds_the_listed_tiles_and_nothing_else():
    rng, sh, pt, k, v, q, d_o, sel, cnt = _problem(3)
    table, n_union = oracle.offload_stage_table(sh, sel, cnt)
    sdk = rng.standard_normal((n_union, sh.Hkv, sh.P, sh.D)).astype(np.float32)
    sdv = rng.standard_normal(sdk.shape).astype(np.float32)
    hk0 = rng.standard_normal(k.shape).astype(np.float32)
    hv0 = rng.standard_normal(k.shape).astype(np.float32)
    hk, hv = oracle.offload_writeback(sh, sdk, sdv, hk0, hv0, pt, sel, cnt)
    touched = np.zeros(k.shape[:2], bool)
    for g in range(sh.Hkv):
        for l in sel[g, : cnt[g]]:
            touched[pt[l], g] = True
            assert np.array_equal(hk[pt[l], g], hk0[pt[l], g] + sdk[table[l], g])
            assert np.array_equal(hv[pt[l], g], hv0[pt[l], g] + sdv[table[l], g])
    assert np.array_equal(hk[~touched], hk0[~touched]) and np.array_equal(hv[~touched], hv0[~touched])


def test_writeback_adds_a_tile_once_however_many_lists_hold_its_page():
    rng, sh, pt, k, v, q, d_o, sel, cnt = _problem(8)
    sel3, cnt3 = _qp_lists(rng, sh)      # the local page n_past is in every list of a head
    table, n_union = oracle.offload_stage_table(sh, sel3, cnt3)
    ones = np.ones((n_union, sh.Hkv, sh.P, sh.D), np.float32)
    hk, hv = oracle.offload_writeback(sh, ones, ones, np.zeros_like(k), np.zeros_like(k), pt, sel3, cnt3)
    assert set(np.unique(hk)) <= {0.0, 1.0} and hk[pt[sh.n_past], 0].min() == 1.0


def test_attention_over_the_staged_pages_is_the_attention_over_the_resident_pool():
    rng, sh, pt, k, v, q, d_o, sel, cnt = _problem(4)
    ref = oracle.attn_fwd_bwd(sh, q, k, v, pt, d_o, sel, cnt, prec="f32")
    table, n_union = oracle.offload_stage_table(sh, sel, cnt)
    shape = (n_union, sh.Hkv, sh.P, sh.D)
    nan = np.full(shape, np.nan, np.float32)       # tiles that are never fetched must never be read
    sk, sv = oracle.offload_fetch(sh, k, v, pt, sel, cnt, nan, nan)
    # (pages in no list keep -1 in the table: attention must never look them up)
    got = oracle.attn_fwd_bwd(sh, q, sk, sv, table, d_o, sel, cnt, prec="f32")
    for key in ("o", "lse", "dq"):
        assert np.array_equal(got[key], ref[key]), key
    hk, hv = oracle.offload_writeback(sh, got["dk_pool"], got["dv_pool"], np.zeros_like(k), np.zeros_like(k), pt, sel, cnt)
    assert np.array_equal(hk, ref["dk_pool"]) and np.array_equal(hv, ref["dv_pool"])


def test_staged_attention_with_per_query_page_lists():
    rng, sh, pt, k, v, q, d_o, sel, cnt = _problem(6)
    sel3, cnt3 = _qp_lists(rng, sh)
    ref = oracle.attn_fwd_bwd(sh, q, k, v, pt, d_o, sel3, cnt3, prec="f32")
    table, n_union = oracle.offload_stage_table(sh, sel3, cnt3)
    nan = np.full((n_union, sh.Hkv, sh.P, sh.D), np.nan, np.float32)
    sk, sv = oracle.offload_fetch(sh, k, v, pt, sel3, cnt3, nan, nan)
    got = oracle.attn_fwd_bwd(sh, q, sk, sv, table, d_o, sel3, cnt3, prec="f32")
    for key in ("o", "lse", "dq"):
        assert np.array_equal(got[key], ref[key]), key
    hk, hv = oracle.offload_writeback(sh, got["dk_pool"], got["dv_pool"], np.zeros_like(k), np.zeros_like(k), pt, sel3, cnt3)
    assert np.array_equal(hk, ref["dk_pool"]) and np.array_equal(hv, ref["dv_pool"])
