"""Pins of the oracle's precondition checker: every planted violation raises exactly its bit, valid
inputs raise none."""
import numpy as np

import oracle
from oracle import Shape

SH = Shape(4, 2, 16, 8, 24, 96, 0.25)   # n = 12, m = 3, n_past = 9


def _valid():
    pt = np.array([5, 0, 7, 3, 9, 1, 12, 4, 8, 2, 6, 11], np.int32)
    sel = np.array([[1, 4, 9, 10, 11], [0, 2, 9, 10, 11]], np.int32)
    cnt = np.array([5, 5], np.int32)
    return pt, sel, cnt


def test_valid_inputs_raise_nothing():
    pt, sel, cnt = _valid()
    assert oracle.check_inputs(SH, 13, pt) == 0
    assert oracle.check_inputs(SH, 13, pt, sel, cnt) == 0
    sel3 = np.full((2, 3, 5), -1, np.int32)
    cnt3 = np.zeros((2, 3), np.int32)
    for g in range(2):
        for tau in range(3):
            lst = [g, 5] + list(range(9, 10 + tau))
            sel3[g, tau, : len(lst)] = lst
            cnt3[g, tau] = len(lst)
    assert oracle.check_inputs(SH, 13, pt, sel3, cnt3) == 0
    # a list per query page may stop at its own local page; without it the bit is raised
    sel3[1, 2, :4] = [1, 5, 9, 10]
    cnt3[1, 2] = 4
    assert oracle.check_inputs(SH, 13, pt, sel3, cnt3) == oracle.CHECK_LIST_LOCAL


def test_each_violation_raises_its_bit():
    pt, sel, cnt = _valid()
    p2 = pt.copy(); p2[3] = 13
    assert oracle.check_inputs(SH, 13, p2, sel, cnt) == oracle.CHECK_TABLE_RANGE
    p2 = pt.copy(); p2[3] = pt[8]
    assert oracle.check_inputs(SH, 13, p2, sel, cnt) == oracle.CHECK_TABLE_DISTINCT
    c2 = cnt.copy(); c2[1] = 6
    assert oracle.check_inputs(SH, 13, pt, sel, c2) == oracle.CHECK_LIST_COUNT
    s2 = sel.copy(); s2[0, 1] = 12; s2[0, 2:] = [13, 14, 15]
    assert oracle.check_inputs(SH, 13, pt, s2, cnt) & oracle.CHECK_LIST_RANGE
    s2 = sel.copy(); s2[0, :2] = [4, 1]
    assert oracle.check_inputs(SH, 13, pt, s2, cnt) == oracle.CHECK_LIST_ORDER
    s2 = sel.copy(); s2[0, :2] = [4, 4]
    assert oracle.check_inputs(SH, 13, pt, s2, cnt) == oracle.CHECK_LIST_ORDER
    s2 = sel.copy(); s2[1] = [0, 2, 3, 10, 11]
    assert oracle.check_inputs(SH, 13, pt, s2, cnt) == oracle.CHECK_LIST_LOCAL
    # entries behind the count are not looked at
    s2 = sel.copy(); c2 = cnt.copy()
    s2 = np.concatenate([s2, np.full((2, 2), 99, np.int32)], axis=1)
    assert oracle.check_inputs(SH, 13, pt, s2, c2) == 0
