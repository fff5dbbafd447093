"""Pins for the CPU oracle's page scoring + top-k (Sec. 4.2; CPU only)."""
import numpy as np
import pytest
import torch

from oracle import Shape


def _problem(sh, seed, extra=2):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((sh.C, sh.Hq, sh.D)).astype(np.float32)
    k = rng.standard_normal((sh.n + extra, sh.Hkv, sh.P, sh.D)).astype(np.float32)
    pt = rng.permutation(sh.n + extra).astype(np.int32)
    return q, k, pt


def _scores_f64(sh, q, k, pt):
    """Mean-pooled chunk query . mean-pooled page key, per KV head, in float64."""
    qg = q.astype(np.float64).reshape(sh.C, sh.Hkv, sh.G, sh.D).mean(axis=(0, 2))       # [Hkv][D]
    kbar = k.astype(np.float64)[pt[:sh.n_past]].mean(axis=2)                            # [n_past][Hkv][D]
    return np.einsum("gd,lgd->gl", qg, kbar)


def _brute_force_select(scores_g, k_eff):
    order = sorted(range(len(scores_g)), key=lambda l: (-float(scores_g[l]), l))
    return sorted(order[:k_eff])


SH = [Shape(Hq=4, Hkv=2, D=8, P=4, C=8, N=64, sm_scale=1.0),
      Shape(Hq=6, Hkv=2, D=16, P=8, C=16, N=256, sm_scale=1.0),
      Shape(Hq=2, Hkv=1, D=64, P=16, C=128, N=1024, sm_scale=0.125)]


@pytest.mark.parametrize("sh", SH)
def test_scores_match_float64_definition(oracle, sh):
    q, k, pt = _problem(sh, 1)
    _, _, scores = oracle.page_score_topk(sh, q, k, pt, top_k=3)
    ref = _scores_f64(sh, q, k, pt)
    assert scores.shape == ref.shape
    assert np.abs(scores - ref).max() < 1e-5 * max(1.0, np.abs(ref).max())


def test_score_of_exactly_representable_inputs_is_exact(oracle):
    """Small integers: every partial sum is exact in fp32, so any summation
    order gives the same bits as the float64 definition."""
    sh = Shape(Hq=4, Hkv=2, D=8, P=4, C=8, N=64, sm_scale=1.0)
    rng = np.random.default_rng(2)
    q = rng.integers(-3, 4, size=(sh.C, sh.Hq, sh.D)).astype(np.float32)
    k = rng.integers(-3, 4, size=(sh.n, sh.Hkv, sh.P, sh.D)).astype(np.float32)
    pt = rng.permutation(sh.n).astype(np.int32)
    _, _, scores = oracle.page_score_topk(sh, q, k, pt, top_k=3)
    ref = _scores_f64(sh, q, k, pt)          # C*G = 16 and P = 4 are powers of two: exact
    assert np.array_equal(scores.astype(np.float64), ref)


@pytest.mark.parametrize("sh", SH)
@pytest.mark.parametrize("top_k", [1, 3, 7])
def test_topk_against_brute_force(oracle, sh, top_k):
    q, k, pt = _problem(sh, 3)
    sel, cnt, scores = oracle.page_score_topk(sh, q, k, pt, top_k=top_k)
    for g in range(sh.Hkv):
        k_eff = min(top_k, sh.n_past)
        want = _brute_force_select(scores[g], k_eff) + list(range(sh.n_past, sh.n))
        assert cnt[g] == len(want)
        assert list(sel[g][:cnt[g]]) == want
        assert np.all(sel[g][cnt[g]:] == -1)
        chosen = scores[g][sel[g][:k_eff]]
        rest = np.delete(scores[g], sel[g][:k_eff])
        assert chosen.min() >= rest.max()


def test_topk_larger_than_history_selects_everything(oracle):
    sh = SH[0]
    q, k, pt = _problem(sh, 4)
    sel, cnt, _ = oracle.page_score_topk(sh, q, k, pt, top_k=sh.n_past + 5)
    for g in range(sh.Hkv):
        assert cnt[g] == sh.n
        assert list(sel[g][:sh.n]) == list(range(sh.n))


def test_no_history(oracle):
    sh = Shape(Hq=4, Hkv=2, D=8, P=4, C=8, N=8, sm_scale=1.0)
    q, k, pt = _problem(sh, 5)
    sel, cnt, scores = oracle.page_score_topk(sh, q, k, pt, top_k=3)
    assert scores.shape == (2, 0)
    for g in range(2):
        assert cnt[g] == 2 and list(sel[g][:2]) == [0, 1]


def test_ties_go_to_the_lower_logical_id(oracle):
    """Pages with identical keys have identical scores; the lower logical id wins
    regardless of where the pages sit physically; -0 and +0 tie as well."""
    sh = SH[0]
    q, k, pt = _problem(sh, 6)
    # make logical pages 3, 9, 11 copies of one page
    for l in (9, 11):
        k[pt[l]] = k[pt[3]]
    sel, cnt, scores = oracle.page_score_topk(sh, q, k, pt, top_k=sh.n_past)
    assert np.all(scores[:, 3] == scores[:, 9]) and np.all(scores[:, 3] == scores[:, 11])
    for g in range(sh.Hkv):
        rank = sorted(range(sh.n_past), key=lambda l: (-float(scores[g][l]), l))
        pos = rank.index(3)
        # choose k so that exactly one / two of the three tied pages fit
        for extra, want in ((1, [3]), (2, [3, 9])):
            s, c, _ = oracle.page_score_topk(sh, q, k, pt, top_k=pos + extra)
            got = [l for l in s[g][:c[g]] if l in (3, 9, 11)]
            assert got == want
    # all-zero keys: every score is +0 or -0, which compare equal -> lowest ids
    k0 = np.zeros_like(k)
    k0[pt[5]] = -0.0
    s, c, sc = oracle.page_score_topk(sh, q, k0, pt, top_k=4)
    assert not sc.any()
    for g in range(sh.Hkv):
        assert list(s[g][:4]) == [0, 1, 2, 3]


def test_selection_placement_invariance(oracle):
    sh = SH[1]
    q, k, pt = _problem(sh, 7)
    a = oracle.page_score_topk(sh, q, k, pt, top_k=5)
    perm = np.random.default_rng(8).permutation(k.shape[0])
    k2 = np.empty_like(k)
    k2[perm] = k
    b = oracle.page_score_topk(sh, q, k2, perm[pt].astype(np.int32), top_k=5)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_boosted_pages_are_retrieved(oracle):
    """Keys offset along the pooled query direction must win the top-k."""
    sh = SH[2]
    q, k, pt = _problem(sh, 9)
    qbar = q.reshape(sh.C, sh.Hkv, sh.G, sh.D).mean(axis=(0, 2))[0]
    boosted = [5, 17, 40]
    for l in boosted:
        k[pt[l], 0] += 4.0 * np.sign(qbar)[None, :]
    sel, cnt, _ = oracle.page_score_topk(sh, q, k, pt, top_k=3)
    assert list(sel[0][:3]) == boosted


def test_bf16_inputs(oracle):
    sh = SH[1]
    q, k, pt = _problem(sh, 10)
    qb = torch.tensor(q).to(torch.bfloat16)
    kb = torch.tensor(k).to(torch.bfloat16)
    a = oracle.page_score_topk(sh, qb.view(torch.int16).numpy().view(np.uint16),
                               kb.view(torch.int16).numpy().view(np.uint16), pt, top_k=4)
    b = oracle.page_score_topk(sh, qb.float().numpy(), kb.float().numpy(), pt, top_k=4)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
