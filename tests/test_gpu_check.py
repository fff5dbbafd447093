"""The device-side checker of the documented preconditions against the oracle's: valid inputs raise
nothing, every planted violation raises its bit.  (The violations are planted in the inputs of the
checker only; it reads them without dereferencing an unchecked index.)"""
import numpy as np
import pytest
import torch

from paper_2602_02108_amd import api
from paper_2602_02108_amd.workloads import WORKLOADS, make_inputs, torch_dtype

import oracle as orc
import parity_util as pu
from test_gpu_qp_attention import rand_qp_lists

pytestmark = pytest.mark.gpu


def _both(w, desc, pt, sel=None, cnt=None):
    got = api.check_inputs(desc, torch.as_tensor(pt, device="cuda"),
                           None if sel is None else torch.as_tensor(sel, device="cuda"),
                           None if cnt is None else torch.as_tensor(cnt, device="cuda"))
    want = orc.check_inputs(pu.shape_of(w), w.n_phys, pt, sel, cnt)
    assert got == want, (got, want)
    return got


def test_checker_matches_the_oracle():
    w = WORKLOADS["mid_sparse_bf16"]
    x = make_inputs(w, "cuda")
    desc = api.make_desc(x["q"], x["k_pool"], w.N, w.sm_scale, torch_dtype(w.grad_dtype))
    sel, cnt, _ = pu.gpu_select(w, x)
    pt = x["page_table"].cpu().numpy()
    sel, cnt = sel.cpu().numpy(), cnt.cpu().numpy()
    assert _both(w, desc, pt) == 0
    assert _both(w, desc, pt, sel, cnt) == 0                       # what the selection kernel emits is valid
    qsel, qcnt = rand_qp_lists(w, 5, 71, popular=2)
    assert _both(w, desc, pt, qsel, qcnt) == 0

    p2 = pt.copy(); p2[3] = w.n_phys
    assert _both(w, desc, p2, sel, cnt) == orc.CHECK_TABLE_RANGE
    p2 = pt.copy(); p2[3] = -1
    assert _both(w, desc, p2) == orc.CHECK_TABLE_RANGE
    p2 = pt.copy(); p2[5] = pt[17]
    assert _both(w, desc, p2, sel, cnt) == orc.CHECK_TABLE_DISTINCT
    c2 = cnt.copy(); c2[2] = sel.shape[1] + 1
    assert _both(w, desc, pt, sel, c2) & orc.CHECK_LIST_COUNT
    s2 = sel.copy(); s2[1, 0] = -3
    assert _both(w, desc, pt, s2, cnt) & orc.CHECK_LIST_RANGE
    s2 = sel.copy(); s2[0, 0], s2[0, 1] = sel[0, 1], sel[0, 0]
    assert _both(w, desc, pt, s2, cnt) == orc.CHECK_LIST_ORDER
    s2 = sel.copy(); s2[3, cnt[3] - 1] = -1; c2 = cnt.copy(); c2[3] -= 1      # the last local page dropped
    assert _both(w, desc, pt, s2, c2) == orc.CHECK_LIST_LOCAL
    q2 = qsel.copy(); c2 = qcnt.copy(); c2[1, 2] -= 1                         # query page 2 without its own page
    assert _both(w, desc, pt, q2, c2) == orc.CHECK_LIST_LOCAL
