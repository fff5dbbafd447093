"""Pins of the oracle's paged-manager steps either side of the attention path (paper Sec. 4.1:
pages are appended chunk by chunk; Sec. 4.2: local-attention layers retrieve the most recent
pages) and of the selection that reads cached page means.  Checked against independent code:
placement by direct indexing, means by an explicit sequential float32 loop, the cached selection
against the streaming one (pinned by brute force elsewhere), the local list by its closed form."""
import numpy as np
import pytest

import oracle
from oracle import Shape


def _problem(seed, Hq=4, Hkv=2, D=64, P=16, C=32, N=160, extra_phys=3):
    rng = np.random.default_rng(seed)
    sh = Shape(Hq, Hkv, D, P, C, N, 1.0 / np.sqrt(D))
    n_phys = sh.n + extra_phys
    page_table = rng.permutation(n_phys)[: sh.n].astype(np.int32)
    k_pool = rng.standard_normal((n_phys, Hkv, P, D)).astype(np.float32)
    v_pool = rng.standard_normal((n_phys, Hkv, P, D)).astype(np.float32)
    q = rng.standard_normal((C, Hq, D)).astype(np.float32)
    return rng, sh, page_table, k_pool, v_pool, q


def _seq_mean(rows):
    """Left-to-right float32 sum of the rows, then one multiply by 1/P (P a power of two)."""
    acc = np.zeros(rows.shape[1], dtype=np.float32)
    for r in rows:
        acc = (acc + r.astype(np.float32)).astype(np.float32)
    return (acc * np.float32(1.0 / rows.shape[0])).astype(np.float32)


def test_append_places_every_chunk_token_and_touches_nothing_else():
    rng, sh, pt, k_pool, v_pool, _ = _problem(1)
    kc = rng.standard_normal((sh.C, sh.Hkv, sh.D)).astype(np.float32)
    vc = rng.standard_normal((sh.C, sh.Hkv, sh.D)).astype(np.float32)
    k2, v2, _ = oracle.kv_append(sh, kc, vc, pt, k_pool, v_pool)
    touched = set()
    for i in range(sh.C):
        phys = pt[sh.n_past + i // sh.P]
        touched.add(int(phys))
        for g in range(sh.Hkv):
            assert np.array_equal(k2[phys, g, i % sh.P], kc[i, g])
            assert np.array_equal(v2[phys, g, i % sh.P], vc[i, g])
    for phys in range(k_pool.shape[0]):
        if phys not in touched:
            assert np.array_equal(k2[phys], k_pool[phys]) and np.array_equal(v2[phys], v_pool[phys])
    assert len(touched) == sh.m


def test_append_writes_the_sequential_means_of_the_new_pages_only():
    rng, sh, pt, k_pool, v_pool, _ = _problem(2)
    kc = rng.standard_normal((sh.C, sh.Hkv, sh.D)).astype(np.float32)
    vc = rng.standard_normal((sh.C, sh.Hkv, sh.D)).astype(np.float32)
    cache0 = rng.standard_normal((sh.n, sh.Hkv, sh.D)).astype(np.float32)
    _, _, cache = oracle.kv_append(sh, kc, vc, pt, k_pool, v_pool, cache0)
    assert np.array_equal(cache[: sh.n_past], cache0[: sh.n_past])
    for tau in range(sh.m):
        for g in range(sh.Hkv):
            want = _seq_mean(kc[tau * sh.P:(tau + 1) * sh.P, g])
            assert np.array_equal(cache[sh.n_past + tau, g].view(np.uint32), want.view(np.uint32))


def test_mean_of_a_constant_page_is_that_token():
    rng, sh, pt, k_pool, v_pool, _ = _problem(3)
    tok = rng.standard_normal((sh.Hkv, sh.D)).astype(np.float32)
    kc = np.broadcast_to(tok, (sh.C, sh.Hkv, sh.D)).copy()
    _, _, cache = oracle.kv_append(sh, kc, kc, pt, k_pool, v_pool, np.zeros((sh.n, sh.Hkv, sh.D), np.float32))
    # P equal summands and a division by P (a power of two): off by at most the P - 1 roundings of the running sum
    for tau in range(sh.m):
        assert np.allclose(cache[sh.n_past + tau], tok, rtol=sh.P * 6e-8, atol=0)


def test_page_means_matches_the_sequential_loop_and_bf16_inputs():
    rng, sh, pt, k_pool, _, _ = _problem(4)
    cache = oracle.page_means(sh, k_pool, pt, 2, 5, np.zeros((sh.n, sh.Hkv, sh.D), np.float32))
    for l in range(sh.n):
        for g in range(sh.Hkv):
            want = _seq_mean(k_pool[pt[l], g]) if 2 <= l < 7 else np.zeros(sh.D, np.float32)
            assert np.array_equal(cache[l, g].view(np.uint32), want.view(np.uint32))
    # bf16 bit patterns: exact conversion to float32 before the sums
    kb = (k_pool.view(np.uint32) >> 16).astype(np.uint16)
    kf = (kb.astype(np.uint32) << 16).view(np.float32)
    cache_b = oracle.page_means(sh, kb, pt, 0, sh.n, np.zeros((sh.n, sh.Hkv, sh.D), np.float32))
    cache_f = oracle.page_means(sh, kf, pt, 0, sh.n, np.zeros((sh.n, sh.Hkv, sh.D), np.float32))
    assert np.array_equal(cache_b.view(np.uint32), cache_f.view(np.uint32))


@pytest.mark.parametrize("seed,top_k", [(5, 3), (6, 0), (7, 100)])
def test_cached_selection_equals_the_streaming_selection_bit_for_bit(seed, top_k):
    rng, sh, pt, k_pool, _, q = _problem(seed)
    cache = oracle.page_means(sh, k_pool, pt, 0, sh.n_past, np.zeros((sh.n, sh.Hkv, sh.D), np.float32))
    sel_s, cnt_s, sc_s = oracle.page_score_topk(sh, q, k_pool, pt, top_k)
    sel_c, cnt_c, sc_c = oracle.page_score_topk_cached(sh, q, cache, top_k)
    assert np.array_equal(sc_s.view(np.uint32), sc_c.view(np.uint32))
    assert np.array_equal(sel_s, sel_c) and np.array_equal(cnt_s, cnt_c)


def test_cached_selection_reads_the_cache_not_the_keys():
    rng, sh, pt, k_pool, _, q = _problem(8)
    cache = oracle.page_means(sh, k_pool, pt, 0, sh.n_past, np.zeros((sh.n, sh.Hkv, sh.D), np.float32))
    # make one page the obvious winner through the cache alone
    qbar = q.reshape(sh.C, sh.Hkv, sh.G, sh.D).mean(axis=(0, 2))
    cache[3] = 50.0 * qbar / np.linalg.norm(qbar, axis=-1, keepdims=True)
    sel, cnt, _ = oracle.page_score_topk_cached(sh, q, cache, 1)
    assert all(int(sel[g][0]) == 3 for g in range(sh.Hkv))


def test_append_then_next_chunk_scores_use_the_appended_means():
    """Chunk recurrence: after chunk c is appended its pages are past pages of chunk c + 1."""
    rng, sh, pt, k_pool, v_pool, q = _problem(9, N=160 - 32)          # context before the append: 4 pages + chunk
    kc = rng.standard_normal((sh.C, sh.Hkv, sh.D)).astype(np.float32)
    cache = oracle.page_means(sh, k_pool, pt, 0, sh.n_past, np.zeros((sh.n + sh.m, sh.Hkv, sh.D), np.float32))
    k2, v2, cache = oracle.kv_append(sh, kc, kc, pt, k_pool, v_pool, cache)
    nxt = Shape(sh.Hq, sh.Hkv, sh.D, sh.P, sh.C, sh.N + sh.C, sh.sm_scale)
    pt2 = np.concatenate([pt, np.setdiff1d(np.arange(k_pool.shape[0]), pt)[: sh.m].astype(np.int32)])
    a = oracle.page_score_topk(nxt, q, k2, pt2, 2)
    b = oracle.page_score_topk_cached(nxt, q, cache, 2)
    assert np.array_equal(a[2].view(np.uint32), b[2].view(np.uint32)) and np.array_equal(a[0], b[0])


@pytest.mark.parametrize("window", [0, 1, 3, 8, 50])
def test_local_page_list_closed_form(window):
    sh = Shape(4, 2, 64, 16, 32, 160, 0.125)
    sel, cnt = oracle.local_page_list(sh, window)
    w = min(window, sh.n_past)
    want = list(range(sh.n_past - w, sh.n))
    for g in range(sh.Hkv):
        assert cnt[g] == w + sh.m
        assert sel[g][: cnt[g]].tolist() == want
        assert (sel[g][cnt[g]:] == -1).all()


def test_local_list_attention_equals_dense_attention_over_a_truncated_context():
    """Attending the last w past pages + the chunk is dense attention over a context that starts w pages back."""
    rng, sh, pt, k_pool, v_pool, q = _problem(10)
    w = 3
    sel, cnt = oracle.local_page_list(sh, w)
    o, lse = oracle.attn_fwd(sh, q, k_pool, v_pool, pt, sel, cnt)
    short = Shape(sh.Hq, sh.Hkv, sh.D, sh.P, sh.C, (w + sh.m) * sh.P, sh.sm_scale)
    o2, lse2 = oracle.attn_fwd(short, q, k_pool, v_pool, pt[sh.n_past - w:])
    assert np.allclose(o, o2, rtol=1e-5, atol=1e-6) and np.allclose(lse, lse2, rtol=1e-5, atol=1e-6)
