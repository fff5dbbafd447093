"""Pins for the CPU oracle's attention forward / backward (CPU only).

The oracle is checked against things other than itself: finite differences, a
library routine (torch SDPA + autograd with an explicit mask), closed forms,
and invariants the method must satisfy (placement invariance, chunk
composition per Sec. 3 Eq. 3, untouched pages per Sec. 4.1).
"""
import math

import numpy as np
import pytest
import torch

from oracle import Shape


def _rand_problem(sh, seed, extra_phys=3, dtype=np.float64):
    rng = np.random.default_rng(seed)
    n_phys = sh.n + extra_phys
    q = rng.standard_normal((sh.C, sh.Hq, sh.D)).astype(dtype)
    d_o = rng.standard_normal((sh.C, sh.Hq, sh.D)).astype(dtype)
    k = rng.standard_normal((n_phys, sh.Hkv, sh.P, sh.D)).astype(dtype)
    v = rng.standard_normal((n_phys, sh.Hkv, sh.P, sh.D)).astype(dtype)
    pt = rng.permutation(n_phys).astype(np.int32)
    return q, d_o, k, v, pt


def _rand_sel(sh, k_sel, seed):
    """A valid list per KV head: k_sel distinct past pages + the m local pages, ascending."""
    rng = np.random.default_rng(seed)
    sel = np.full((sh.Hkv, k_sel + sh.m), -1, dtype=np.int32)
    for g in range(sh.Hkv):
        past = np.sort(rng.choice(sh.n_past, size=k_sel, replace=False))
        sel[g] = np.concatenate([past, np.arange(sh.n_past, sh.n)])
    cnt = np.full(sh.Hkv, k_sel + sh.m, dtype=np.int32)
    return sel, cnt


def _flatten(sh, pool, pt):
    """[N][Hkv][D] logical-order view of a pool (test-side helper)."""
    return pool[pt[:sh.n]].transpose(0, 2, 1, 3).reshape(sh.N, sh.Hkv, sh.D)


def _mask(sh, sel):
    """Boolean [Hkv][C][N] visibility from the definition: page selected and t <= a_i."""
    msk = np.zeros((sh.Hkv, sh.C, sh.N), dtype=bool)
    a = sh.N - sh.C + np.arange(sh.C)
    t = np.arange(sh.N)
    causal = t[None, :] <= a[:, None]
    for g in range(sh.Hkv):
        pages = np.arange(sh.n) if sel is None else sel[g][sel[g] >= 0]
        page_ok = np.isin(t // sh.P, pages)
        msk[g] = causal & page_ok[None, :]
    return msk


def _torch_reference(sh, q, d_o, k, v, pt, sel):
    """Library special case: SDPA + autograd on the flattened history with a mask."""
    kf = torch.tensor(_flatten(sh, k, pt), dtype=torch.float64, requires_grad=True)
    vf = torch.tensor(_flatten(sh, v, pt), dtype=torch.float64, requires_grad=True)
    qt = torch.tensor(q, dtype=torch.float64, requires_grad=True)
    msk = torch.tensor(_mask(sh, sel))                       # [Hkv][C][N]
    msk_h = msk.repeat_interleave(sh.G, dim=0)               # [Hq][C][N]
    qh = qt.permute(1, 0, 2)                                  # [Hq][C][D]
    kh = kf.permute(1, 0, 2).repeat_interleave(sh.G, dim=0)   # [Hq][N][D]
    vh = vf.permute(1, 0, 2).repeat_interleave(sh.G, dim=0)
    o = torch.nn.functional.scaled_dot_product_attention(qh, kh, vh, attn_mask=msk_h, scale=sh.sm_scale)
    logits = (qh @ kh.transpose(1, 2)) * sh.sm_scale
    lse = torch.logsumexp(logits.masked_fill(~msk_h, -math.inf), dim=-1)
    o.backward(torch.tensor(d_o, dtype=torch.float64).permute(1, 0, 2))
    return (o.permute(1, 0, 2).detach().numpy(), lse.detach().numpy(), qt.grad.numpy(),
            kf.grad.numpy(), vf.grad.numpy())


def _unflatten_grad(sh, pool_grad, pt):
    """Pool-shaped gradient -> [N][Hkv][D] logical order."""
    return _flatten(sh, pool_grad, pt)


SHAPES = [
    Shape(Hq=4, Hkv=2, D=8, P=4, C=8, N=32, sm_scale=0.3),
    Shape(Hq=6, Hkv=2, D=16, P=8, C=16, N=64, sm_scale=0.25),
    Shape(Hq=2, Hkv=1, D=64, P=16, C=128, N=1024, sm_scale=0.125),   # tiny config of the benchmark set
]


@pytest.mark.parametrize("sh", SHAPES[:2])
@pytest.mark.parametrize("sparse", [False, True])
def test_finite_differences(oracle, sh, sparse):
    q, d_o, k, v, pt = _rand_problem(sh, 1)
    sel, cnt = _rand_sel(sh, 2, 2) if sparse else (None, None)
    res = oracle.attn_fwd_bwd(sh, q, k, v, pt, d_o, sel, cnt, prec="f64")

    def loss(q_, k_, v_):
        o, _ = oracle.attn_fwd(sh, q_, k_, v_, pt, sel, cnt, prec="f64")
        return float((o * d_o).sum())

    rng = np.random.default_rng(3)
    eps = 1e-5
    for name, arr, grad in (("q", q, res["dq"]), ("k", k, res["dk_pool"]), ("v", v, res["dv_pool"])):
        nz = np.argwhere(grad != 0)
        picks = nz[rng.choice(len(nz), size=12, replace=False)]
        # also probe entries whose gradient must be exactly zero (unselected / unreferenced pages)
        z = np.argwhere(grad == 0)
        if len(z):
            picks = np.concatenate([picks, z[rng.choice(len(z), size=min(4, len(z)), replace=False)]])
        for idx in picks:
            idx = tuple(idx)
            args = dict(q=q.copy(), k=k.copy(), v=v.copy())
            args[name][idx] += eps
            lp = loss(args["q"], args["k"], args["v"])
            args[name][idx] -= 2 * eps
            lm = loss(args["q"], args["k"], args["v"])
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad[idx]) <= 1e-6 * max(1.0, abs(grad[idx])), (name, idx, fd, grad[idx])


@pytest.mark.parametrize("sh", SHAPES)
@pytest.mark.parametrize("sparse", [False, True])
@pytest.mark.parametrize("prec,tol", [("f64", 1e-10), ("f32", 2e-5)])
def test_against_library_sdpa_autograd(oracle, sh, sparse, prec, tol):
    q, d_o, k, v, pt = _rand_problem(sh, 11)
    sel, cnt = _rand_sel(sh, min(3, sh.n_past), 12) if sparse else (None, None)
    res = oracle.attn_fwd_bwd(sh, q, k, v, pt, d_o, sel, cnt, prec=prec)
    o, lse, dq, dkf, dvf = _torch_reference(sh, q, d_o, k, v, pt, sel)

    def rel(a, b):
        return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30)

    assert rel(res["o"], o) < tol
    assert rel(res["lse"], lse) < tol
    assert rel(res["dq"], dq) < tol
    assert rel(_unflatten_grad(sh, res["dk_pool"], pt), dkf) < tol
    assert rel(_unflatten_grad(sh, res["dv_pool"], pt), dvf) < tol
    # physical pages that the page table's first n entries never reference stay zero
    unref = np.setdiff1d(np.arange(k.shape[0]), pt[:sh.n])
    assert not res["dk_pool"][unref].any() and not res["dv_pool"][unref].any()


def test_row_subset_matches_full(oracle):
    sh = SHAPES[1]
    q, d_o, k, v, pt = _rand_problem(sh, 21)
    sel, cnt = _rand_sel(sh, 3, 22)
    full = oracle.attn_fwd_bwd(sh, q, k, v, pt, d_o, sel, cnt, prec="f64")
    rows = np.array([[0, 0], [5, 15], [3, 7], [2, 8]], dtype=np.int32)
    o, lse = oracle.attn_fwd(sh, q, k, v, pt, sel, cnt, rows=rows, prec="f64")
    dq = oracle.attn_bwd_dq(sh, q, k, v, pt, full["lse"], full["delta"], d_o, sel, cnt, rows=rows, prec="f64")
    for r, (h, i) in enumerate(rows):
        assert np.array_equal(o[r], full["o"][i, h])
        assert lse[r] == full["lse"][h, i]
        assert np.array_equal(dq[r], full["dq"][i, h])
    # page-unit subset of dK/dV
    g, l = 1, int(sel[1][1])
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    oracle.attn_bwd_dkv(sh, q, k, v, pt, full["lse"], full["delta"], d_o, dk, dv, sel, cnt,
                        units=np.array([[g, l]]), prec="f64")
    assert np.array_equal(dk[pt[l], g], full["dk_pool"][pt[l], g])
    assert np.array_equal(dv[pt[l], g], full["dv_pool"][pt[l], g])
    dk[pt[l], g] = 0
    dv[pt[l], g] = 0
    assert not dk.any() and not dv.any()
    # a page that is not in the list contributes nothing
    not_sel = int(np.setdiff1d(np.arange(sh.n_past), sel[0])[0])
    oracle.attn_bwd_dkv(sh, q, k, v, pt, full["lse"], full["delta"], d_o, dk, dv, sel, cnt,
                        units=np.array([[0, not_sel]]), prec="f64")
    assert not dk.any() and not dv.any()


def test_closed_form_zero_queries(oracle):
    """Q = 0: O is the mean of the visible V rows and LSE = log(#visible), which
    pins the causal boundary and the visible-set size."""
    sh = SHAPES[1]
    q, d_o, k, v, pt = _rand_problem(sh, 31)
    q[:] = 0
    k_sel = 3
    sel, cnt = _rand_sel(sh, k_sel, 32)
    o, lse = oracle.attn_fwd(sh, q, k, v, pt, sel, cnt, prec="f64")
    vf = _flatten(sh, v, pt)
    for h in range(sh.Hq):
        g = h // sh.G
        for i in range(sh.C):
            count = k_sel * sh.P + i + 1
            assert abs(lse[h, i] - math.log(count)) < 1e-12
            toks = np.concatenate([(p * sh.P + np.arange(sh.P)) for p in sel[g][:k_sel]] +
                                  [np.arange(sh.n_past * sh.P, sh.n_past * sh.P + i + 1)])
            assert np.allclose(o[i, h], vf[toks, g].mean(axis=0), atol=1e-12)


def test_closed_form_constant_values(oracle):
    """V constant over tokens: O equals that constant, dQ = 0 and dK adds nothing."""
    sh = SHAPES[1]
    q, d_o, k, v, pt = _rand_problem(sh, 41)
    const = np.random.default_rng(5).standard_normal((sh.Hkv, sh.D))
    v[:] = const[None, :, None, :]
    sel, cnt = _rand_sel(sh, 2, 42)
    res = oracle.attn_fwd_bwd(sh, q, k, v, pt, d_o, sel, cnt, prec="f64")
    for h in range(sh.Hq):
        assert np.allclose(res["o"][:, h], const[h // sh.G][None, :], atol=1e-12)
    assert np.abs(res["dq"]).max() < 1e-12
    assert np.abs(res["dk_pool"]).max() < 1e-12


def test_row_probabilities_sum_to_one(oracle):
    sh = SHAPES[2]
    q, d_o, k, v, pt = _rand_problem(sh, 51, dtype=np.float32)
    sel, cnt = _rand_sel(sh, 8, 52)
    for prec, tol in (("f32", 1e-5), ("f64", 1e-12)):
        for (h, i) in [(0, 0), (1, 127), (0, 15), (1, 16), (0, 64)]:
            p, tok = oracle.row_probs(sh, q, k, pt, h, i, sel, cnt, prec=prec)
            assert abs(p.sum() - 1.0) < tol
            # visible set: selected pages, nothing beyond the query's own position
            a_i = sh.N - sh.C + i
            assert tok.max() == a_i and len(tok) == 8 * sh.P + i + 1
            assert np.all(np.isin(tok // sh.P, sel[0]))
            assert np.all(np.diff(tok) > 0)


def test_placement_invariance(oracle):
    """Moving pages around physically (and fixing the page table) changes nothing."""
    sh = SHAPES[1]
    q, d_o, k, v, pt = _rand_problem(sh, 61, dtype=np.float32)
    sel, cnt = _rand_sel(sh, 3, 62)
    a = oracle.attn_fwd_bwd(sh, q, k, v, pt, d_o, sel, cnt, prec="f32")
    perm = np.random.default_rng(63).permutation(k.shape[0])     # new_phys = perm[old_phys]
    k2 = np.empty_like(k)
    v2 = np.empty_like(v)
    k2[perm] = k
    v2[perm] = v
    pt2 = perm[pt].astype(np.int32)
    b = oracle.attn_fwd_bwd(sh, q, k2, v2, pt2, d_o, sel, cnt, prec="f32")
    for key in ("o", "lse", "dq"):
        assert np.array_equal(a[key], b[key])
    assert np.array_equal(a["dk_pool"], b["dk_pool"][perm])
    assert np.array_equal(a["dv_pool"], b["dv_pool"][perm])


def test_scale_identity(oracle):
    """S is invariant under Q -> aQ, K -> K/a, hence <dQ, Q> = <dK, K> per KV head."""
    sh = SHAPES[1]
    q, d_o, k, v, pt = _rand_problem(sh, 71)
    sel, cnt = _rand_sel(sh, 3, 72)
    r = oracle.attn_fwd_bwd(sh, q, k, v, pt, d_o, sel, cnt, prec="f64")
    for g in range(sh.Hkv):
        lhs = (r["dq"][:, g * sh.G:(g + 1) * sh.G] * q[:, g * sh.G:(g + 1) * sh.G]).sum()
        rhs = (r["dk_pool"][:, g] * k[:, g]).sum()
        assert abs(lhs - rhs) < 1e-10 * max(1.0, abs(lhs))


def test_chunk_composition(oracle):
    """Sec. 3 Eq. 3: two consecutive chunk calls (dense) accumulate the same
    dK/dV into the pool as one call with a chunk twice as long, and give the same O."""
    one = Shape(Hq=4, Hkv=2, D=8, P=4, C=16, N=40, sm_scale=0.3)
    q, d_o, k, v, pt = _rand_problem(one, 81)
    ref = oracle.attn_fwd_bwd(one, q, k, v, pt, d_o, prec="f64")

    first = Shape(4, 2, 8, 4, 8, 32, 0.3)    # chunk 1: tokens 24..31, history up to 32
    second = Shape(4, 2, 8, 4, 8, 40, 0.3)   # chunk 2: tokens 32..39, history up to 40
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    # backward runs from the last chunk to the first, accumulating into the same pools
    r2 = oracle.attn_fwd_bwd(second, q[8:], k, v, pt, d_o[8:], dk_pool=dk, dv_pool=dv, prec="f64")
    r1 = oracle.attn_fwd_bwd(first, q[:8], k, v, pt, d_o[:8], dk_pool=dk, dv_pool=dv, prec="f64")
    assert np.allclose(np.concatenate([r1["o"], r2["o"]]), ref["o"], atol=1e-12)
    assert np.allclose(np.concatenate([r1["dq"], r2["dq"]]), ref["dq"], atol=1e-12)
    assert np.allclose(dk, ref["dk_pool"], atol=1e-12)
    assert np.allclose(dv, ref["dv_pool"], atol=1e-12)


def test_accumulates_and_leaves_other_pages_untouched(oracle):
    sh = SHAPES[1]
    q, d_o, k, v, pt = _rand_problem(sh, 91)
    sel, cnt = _rand_sel(sh, 2, 92)
    rng = np.random.default_rng(93)
    init_k = rng.standard_normal(k.shape)
    init_v = rng.standard_normal(v.shape)
    zero = oracle.attn_fwd_bwd(sh, q, k, v, pt, d_o, sel, cnt, prec="f64")
    acc = oracle.attn_fwd_bwd(sh, q, k, v, pt, d_o, sel, cnt, dk_pool=init_k.copy(),
                              dv_pool=init_v.copy(), prec="f64")
    assert np.allclose(acc["dk_pool"], init_k + zero["dk_pool"], atol=1e-12)
    assert np.allclose(acc["dv_pool"], init_v + zero["dv_pool"], atol=1e-12)
    for g in range(sh.Hkv):
        touched = pt[sel[g]]
        untouched = np.setdiff1d(np.arange(k.shape[0]), touched)
        assert np.array_equal(acc["dk_pool"][untouched, g], init_k[untouched, g])
        assert np.array_equal(acc["dv_pool"][untouched, g], init_v[untouched, g])


def test_bf16_inputs_are_read_exactly(oracle):
    """bf16 bit patterns in == the same values given as floats."""
    sh = SHAPES[0]
    q, d_o, k, v, pt = _rand_problem(sh, 101, dtype=np.float32)

    def as_bf16(a):
        t = torch.tensor(a).to(torch.bfloat16)
        return t.view(torch.int16).numpy().view(np.uint16), t.float().numpy()

    (qb, qf), (db, df), (kb, kf), (vb, vf) = map(as_bf16, (q, d_o, k, v))
    a = oracle.attn_fwd_bwd(sh, qb, kb, vb, pt, db, prec="f32")
    b = oracle.attn_fwd_bwd(sh, qf, kf, vf, pt, df, prec="f32")
    for key in a:
        assert np.array_equal(a[key], b[key])
