"""Pins for the oracle's row-aware cost variant (no GPU).

The variant charges every level-0 position of an operand `row_cost` units on top of its stored
non-zeros (Section 4.2.2 remarks that the non-zero count only approximates the run time).  It is an
instance of Algorithm 1 (Section 3.2) with another pair of cost functions, so it is pinned like the
plain one: to the properties Section 3.1 demands of cost functions (by enumeration), to the closed
form "the boundary of query Q is the rank-Q item of the sorted list of work items" by brute force
(a row's own units are items at column 0 of that row), to the plain search at row_cost = 0, to the
arithmetic closed form for one CSR operand, and to the tiling invariants.
"""
import numpy as np
import pytest

import oracle
from util import random_coords, to_csr, to_dcsr


def _make(fmt, coords, shape):
    if fmt == "csr":
        pos, crd = to_csr(coords, shape[0])
        return oracle.csr(pos, crd, shape[0], shape[1])
    return oracle.dcsr(*to_dcsr(coords), shape[0], shape[1])


def _items(fmt, coord_lists, shape, rc):
    """Sorted work items of all operands: (row, column) of every entry, and rc items at (row, 0) for
    every row an operand holds a level-0 position for (CSR: every row; DCSR: every stored row)."""
    items = []
    for cl in coord_lists:
        rows = range(shape[0]) if fmt == "csr" else sorted({int(c[0]) for c in cl})
        for i in rows:
            items += [(i, 0)] * rc
        items += [(int(c[0]), int(c[1])) for c in cl]
    return sorted(items)


def _positions(fmt, cl, x):
    rows_before = x[0] if fmt == "csr" else len({int(c[0]) for c in cl if int(c[0]) < x[0]})
    entries_before = sum(1 for c in cl if (int(c[0]), int(c[1])) < tuple(x))
    return [rows_before, entries_before]


@pytest.mark.parametrize("fmt", ["csr", "dcsr"])
@pytest.mark.parametrize("k", [1, 2, 3])
@pytest.mark.parametrize("rc", [1, 3])
def test_rank_q_item(fmt, k, rc):
    rng = np.random.default_rng(100 * k + rc)
    shape = (6, 7)
    for trial in range(10):
        lists = [random_coords(rng, shape, int(rng.integers(0, 25))) for _ in range(k)]
        if trial % 3 == 1 and k > 1:
            lists[1] = lists[0].copy()                       # every coordinate tied
        ops = [_make(fmt, c, shape) for c in lists]
        items = _items(fmt, lists, shape, rc)
        P = len(items) + 1
        parts = oracle.partition_rowcost(ops, P, rc, queries=np.arange(P + 1, dtype=np.int64))
        for Q in range(1, len(items)):
            x = items[Q]
            assert tuple(parts["coord"][Q].tolist()) == x, (fmt, k, rc, trial, Q)
            cost = sum(1 for it in items if it < x)
            assert int(parts["cost"][Q]) == cost
            assert 0 <= Q - cost < k * (rc + 1)              # the tie group at (row, 0) is the largest possible
            for t, cl in enumerate(lists):
                assert parts["posn"][Q, t].tolist() == _positions(fmt, cl, x)


def test_cost_functions_are_monotone_and_hierarchically_consistent():
    """Section 3.1: C is monotone along the lexicographic order, and closing a row adds exactly the
    row's own cost: C(i + 1, 0) - C(i, 0) = sum over operands holding row i of (row_cost + entries)."""
    rng = np.random.default_rng(5)
    shape, rc = (5, 6), 2
    lists = [random_coords(rng, shape, 9), random_coords(rng, shape, 6)]
    for fmt in ("csr", "dcsr"):
        items = _items(fmt, lists, shape, rc)
        C = lambda x: sum(1 for it in items if it < tuple(x))
        prev = -1
        for i in range(shape[0]):
            own = 0
            for cl in lists:
                n_i = sum(1 for c in cl if int(c[0]) == i)
                if fmt == "csr" or n_i > 0:
                    own += rc + n_i
            assert C((i + 1, 0)) - C((i, 0)) == own
            for j in range(shape[1] + 1):
                assert C((i, j)) >= prev
                prev = C((i, j))
        ops = [_make(fmt, c, shape) for c in lists]
        P = len(items) + 1
        parts = oracle.partition_rowcost(ops, P, rc, queries=np.arange(P + 1, dtype=np.int64))
        for Q in range(1, len(items)):
            assert int(parts["cost"][Q]) == C(parts["coord"][Q].tolist())


def test_row_cost_zero_is_the_plain_search():
    rng = np.random.default_rng(9)
    shape = (30, 40)
    for fmt in ("csr", "dcsr"):
        lists = [random_coords(rng, shape, 200), random_coords(rng, shape, 90)]
        ops = [_make(fmt, c, shape) for c in lists]
        for P in (1, 7, 64):
            a = oracle.partition(ops, P)
            b = oracle.partition_rowcost(ops, P, 0)
            for key in ("coord", "posn", "cost"):
                assert np.array_equal(a[key], b[key]), (fmt, P, key)


def test_one_csr_operand_closed_form():
    """One CSR operand: boundary b lies in the row r with pos[r] + rc r <= Q_b < pos[r+1] + rc (r+1); with
    R = Q_b - pos[r] - rc r left, it sits at the row's start when R < rc and at the entry of rank R - rc
    otherwise."""
    rng = np.random.default_rng(13)
    n_rows, n_cols, rc = 50, 60, 2
    c = random_coords(rng, (n_rows, n_cols), 400)
    pos, crd = to_csr(c, n_rows)
    ops = [oracle.csr(pos, crd, n_rows, n_cols)]
    total = int(pos[-1]) + rc * n_rows
    for P in (3, 17, 90):
        parts = oracle.partition_rowcost(ops, P, rc)
        assert int(parts["cost"][-1]) == total
        for b in range(1, P):
            Q = b * total // P
            lo = pos.astype(np.int64)[:-1] + rc * np.arange(n_rows)
            hi = pos.astype(np.int64)[1:] + rc * (np.arange(n_rows) + 1)
            r = int(np.flatnonzero((lo <= Q) & (Q < hi))[0])
            R = Q - int(lo[r])
            at = int(pos[r]) + max(R - rc, 0)
            assert int(parts["coord"][b, 0]) == r and int(parts["posn"][b, 0, 1]) == at
            assert int(parts["posn"][b, 0, 0]) == r
            # (an entry in column 0 shares the coordinate (r, 0) with the row's own units: one tie group)
            x1 = int(crd[at]) if R >= rc else 0
            assert int(parts["coord"][b, 1]) == x1
            assert int(parts["cost"][b]) == int(lo[r]) + (rc + at - int(pos[r]) if x1 > 0 else 0)


def test_tiling_and_balance():
    """Boundaries ordered, position intervals tile the operand, work sums to the total, and no
    partition exceeds its share by more than one tie group."""
    rng = np.random.default_rng(17)
    n_rows, n_cols, rc = 400, 300, 1
    lens = np.minimum(rng.zipf(1.5, n_rows), n_cols)
    c = np.concatenate([np.stack([np.full(l, i), np.sort(rng.choice(n_cols, l, replace=False))], 1)
                        for i, l in enumerate(lens)])
    pos, crd = to_csr(c, n_rows)
    ops = [oracle.csr(pos, crd, n_rows, n_cols)]
    total = int(pos[-1]) + rc * n_rows
    for P in (5, 33):
        parts = oracle.partition_rowcost(ops, P, rc)
        work = np.diff(parts["cost"])
        assert work.sum() == total and work.min() >= 0
        assert work.max() - total / P <= rc + 1
        at = parts["posn"][:, 0, 1]
        assert at[0] == 0 and at[-1] == pos[-1] and np.all(np.diff(at) >= 0)
