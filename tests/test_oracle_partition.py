"""Pins for the oracle's partition search (no GPU).

The oracle follows Algorithm 1 (Section 3.2) with the non-zero-count cost of
Section 4.2.2.  It is pinned here to things other than itself:
  * the two worked examples the paper prints (Figure 2, Figure 3(a));
  * the closed form that follows from monotonicity: for 0 <= Q < Q_total the
    result is the coordinate of the rank-Q element of the sorted merged list of
    all operands' stored coordinates (brute force on tiny inputs);
  * Theorem 1 (Section 3.2.2): 0 <= Q - C(x) < Delta <= number of operands;
  * the tiling invariant (boundaries ordered, position intervals tile every
    operand, work sums to the total);
  * the CSR closed-form cost functions (Section 4.2.2, first listing);
  * numpy's sort / searchsorted on three vectors (the case Section 4.2.3
    specialises), on random inputs.
"""
import json
import os

import numpy as np
import pytest

import oracle
from util import (count_prefix_less, merged_sorted, random_coords, to_csf3, to_csr, to_dcsr,
                  to_vector)


def _load(golden_dir, name):
    with open(os.path.join(golden_dir, name)) as f:
        return json.load(f)


# --------------------------------------------------------------------------- #
# worked examples printed by the paper
# --------------------------------------------------------------------------- #
def test_fig2_three_vectors(golden_dir):
    g = _load(golden_dir, "fig2_three_vector_partition.json")
    ops = [oracle.vector(np.array(g[n], np.int32), g["extent"]) for n in "abc"]
    assert oracle.total_cost(ops) == 12
    parts = oracle.partition(ops, g["P"])
    bounds = parts["coord"][:, 0].tolist()
    assert bounds == [lo for lo, _ in g["partitions"]] + [g["partitions"][-1][1]]
    assert np.diff(parts["cost"]).tolist() == [g["nonzeros_per_partition"]] * g["P"]
    # membership: each operand's entries inside [lo, hi) are exactly the position interval
    for t, n in enumerate("abc"):
        idx = np.array(g[n])
        for p, (lo, hi) in enumerate(g["partitions"]):
            inside = np.flatnonzero((idx >= lo) & (idx < hi))
            got = np.arange(parts["posn"][p, t, 0], parts["posn"][p + 1, t, 0])
            assert inside.tolist() == got.tolist()


def test_fig2_interior_queries_by_literal_search(golden_dir):
    """Interior queries 3, 6, 9 return 2, 5, 10; query 0 returns the first
    occupied coordinate (1), which is why boundary 0 is the origin by definition."""
    g = _load(golden_dir, "fig2_three_vector_partition.json")
    ops = [oracle.vector(np.array(g[n], np.int32), g["extent"]) for n in "abc"]
    assert [int(oracle.find_partition(ops, q)[0][0]) for q in (3, 6, 9)] == [2, 5, 10]
    assert int(oracle.find_partition(ops, 0)[0][0]) == 1
    assert int(oracle.find_partition(ops, 12)[0][0]) == 12


def _dcsr_from_pairs(pairs, n_rows, n_cols):
    c = np.array(pairs, dtype=np.int64)
    p0, c0, p1, c1 = to_dcsr(c)
    return oracle.dcsr(p0, c0, p1, c1, n_rows, n_cols)


def test_fig3a_dcsr_addition(golden_dir):
    g = _load(golden_dir, "fig3a_dcsr_add_partition.json")
    A = _dcsr_from_pairs(g["A"], g["n_rows"], g["n_cols"])
    B = _dcsr_from_pairs(g["B"], g["n_rows"], g["n_cols"])
    parts = oracle.partition([A, B], g["P"])
    assert np.diff(parts["cost"]).tolist() == [6, 6, 6, 6]
    # colours -> number of entries of each operand in each chunk -> positions
    for t, key in enumerate(("A_membership", "B_membership")):
        counts = np.bincount(g[key], minlength=g["P"])
        assert parts["posn"][:, t, 1].tolist() == [0] + np.cumsum(counts).tolist()
    drawn = g["drawn_cuts_row_col"]
    got = parts["coord"][1:-1].tolist()
    assert got[0] == drawn[0] and got[2] == drawn[2]
    # second cut: drawn at the low end of a flat stretch, the search takes the high end
    assert got[1][0] == drawn[1][0] and got[1][1] >= drawn[1][1]
    stored = {tuple(c) for c in g["A"]} | {tuple(c) for c in g["B"]}
    assert all((drawn[1][0], j) not in stored for j in range(drawn[1][1], got[1][1]))
    assert got[1] == [2, 6]
    assert parts["coord"][0].tolist() == [0, 0] and parts["coord"][-1].tolist() == [g["n_rows"], 0]
    # level-0 positions: number of stored rows before the boundary row
    assert parts["posn"][:, 0, 0].tolist() == [0, 0, 1, 2, 3]
    assert parts["posn"][:, 1, 0].tolist() == [0, 0, 1, 2, 3]


# --------------------------------------------------------------------------- #
# closed form: rank-Q element of the merged list; positions and cost by counting
# --------------------------------------------------------------------------- #
def _make(fmt, coords, shape):
    if fmt == "vec":
        return oracle.vector(to_vector(coords), shape[0])
    if fmt == "csr":
        pos, crd = to_csr(coords, shape[0])
        return oracle.csr(pos, crd, shape[0], shape[1])
    if fmt == "dcsr":
        return oracle.dcsr(*to_dcsr(coords), shape[0], shape[1])
    if fmt == "coo":
        return oracle.coo(coords[:, 0].astype(np.int32), coords[:, 1].astype(np.int32), shape[0], shape[1])
    if fmt == "csf3":
        p0, c0, p1, c1, p2, c2 = to_csf3(coords)
        return oracle.Tensor([("compressed", shape[0], p0, c0), ("compressed", shape[1], p1, c1),
                              ("compressed", shape[2], p2, c2)])
    raise ValueError(fmt)


def _brute_boundary(fmt, coord_lists, shape, Q):
    merged = merged_sorted(coord_lists)
    d = len(shape)
    if Q >= len(merged):
        x = (shape[0],) + (0,) * (d - 1)
    else:
        x = merged[Q]
    cost = sum(1 for c in merged if c < x)
    posn = np.zeros((len(coord_lists), d), dtype=np.int64)
    for t, cl in enumerate(coord_lists):
        for m in range(d):
            if fmt == "csr" and m == 0:
                posn[t, m] = x[0]                     # dense level: position == coordinate
            elif fmt == "coo" and m == 0:
                posn[t, m] = sum(1 for c in cl if int(c[0]) < x[0])   # one level-0 entry per non-zero
            else:
                posn[t, m] = count_prefix_less(cl, m, x)
    return x, posn, cost


CASES = [("vec", (40,)), ("csr", (7, 9)), ("dcsr", (9, 7)), ("coo", (9, 7)), ("csf3", (4, 5, 6))]


@pytest.mark.parametrize("fmt,shape", CASES)
@pytest.mark.parametrize("k", [1, 2, 3, 5])
def test_closed_form_rank_q(fmt, shape, k):
    rng = np.random.default_rng(1000 * k + len(shape))
    total = int(np.prod(shape))
    for trial in range(12):
        density = rng.choice([0.0, 0.05, 0.3, 0.9])
        coord_lists = []
        for t in range(k):
            n = int(round(total * density * rng.uniform(0.2, 1.0)))
            if trial % 4 == 1 and t > 0:              # identical operands: every coordinate tied
                coord_lists.append(coord_lists[0].copy())
            else:
                coord_lists.append(random_coords(rng, shape, n))
        ops = [_make(fmt, c, shape) for c in coord_lists]
        qtot = sum(c.shape[0] for c in coord_lists)
        assert oracle.total_cost(ops) == qtot
        for Q in range(0, qtot + 2):
            coord, posn, cost = oracle.find_partition(ops, Q)
            if Q >= qtot:
                assert int(coord[0]) == shape[0]
                continue
            bx, bposn, bcost = _brute_boundary(fmt, coord_lists, shape, Q)
            assert tuple(coord.tolist()) == bx, (fmt, k, trial, Q)
            assert cost == bcost
            assert posn.tolist() == bposn.tolist(), (fmt, k, trial, Q)
            # Theorem 1: 0 <= Q - C(x) < Delta_{d-1} <= k
            assert 0 <= Q - cost < k


@pytest.mark.parametrize("fmt,shape", CASES)
def test_tiling_invariants(fmt, shape):
    rng = np.random.default_rng(77)
    total = int(np.prod(shape))
    for trial in range(10):
        k = int(rng.integers(1, 5))
        coord_lists = [random_coords(rng, shape, int(rng.integers(0, total // 2 + 1))) for _ in range(k)]
        ops = [_make(fmt, c, shape) for c in coord_lists]
        qtot = sum(c.shape[0] for c in coord_lists)
        for P in (1, 2, 3, 7, qtot + 3):
            parts = oracle.partition(ops, P)
            cost, posn, coord = parts["cost"], parts["posn"], parts["coord"]
            assert cost[0] == 0 and cost[-1] == qtot
            assert np.all(np.diff(cost) >= 0) and np.diff(cost).sum() == qtot
            tup = [tuple(c) for c in coord.tolist()]
            assert tup == sorted(tup)
            assert np.all(np.diff(posn, axis=0) >= 0)
            d = len(shape)
            for t in range(k):
                assert posn[-1, t, d - 1] - posn[0, t, d - 1] == coord_lists[t].shape[0]
            # work per partition = entries of all operands between the boundaries
            work = (posn[1:, :, d - 1] - posn[:-1, :, d - 1]).sum(axis=1)
            assert work.tolist() == np.diff(cost).tolist()
            # equally spaced queries: imbalance bounded by the operand count (Theorem 1)
            if qtot > 0:
                q = [(p * qtot) // P for p in range(P + 1)]
                ideal = np.diff(q)
                assert np.all(np.abs(np.diff(cost) - ideal) <= k - 1)


def test_explicit_queries_and_degenerate_inputs():
    rng = np.random.default_rng(5)
    a = random_coords(rng, (50,), 20)
    b = random_coords(rng, (50,), 7)
    ops = [oracle.vector(to_vector(a), 50), oracle.vector(to_vector(b), 50)]
    q = np.array([0, 4, 4, 11, 26, 27, 99], dtype=np.int64)
    parts = oracle.partition(ops, 6, queries=q)
    merged = merged_sorted([a, b])
    for p in (1, 2, 3, 4):
        assert parts["coord"][p, 0] == merged[q[p]][0]
    assert parts["coord"][5, 0] == 50 and parts["coord"][6, 0] == 50    # Q >= total -> end
    # all-empty operands: every boundary after the first is the end
    e = oracle.vector(np.zeros(0, np.int32), 9)
    parts = oracle.partition([e, e], 3)
    assert parts["coord"][:, 0].tolist() == [0, 9, 9, 9] and parts["cost"].tolist() == [0, 0, 0, 0]
    # more partitions than work: repeated boundaries, zero-work partitions
    one = oracle.vector(np.array([4], np.int32), 9)
    parts = oracle.partition([one], 4)
    assert parts["cost"].tolist() == [0, 0, 0, 0, 1]


# --------------------------------------------------------------------------- #
# CSR closed forms (Section 4.2.2): C_i = pos[x_i]-pos[0], C_j = x_jp - pos[x_i]
# --------------------------------------------------------------------------- #
def test_csr_single_operand_closed_form():
    rng = np.random.default_rng(9)
    for trial in range(20):
        n_rows, n_cols = int(rng.integers(1, 30)), int(rng.integers(1, 30))
        c = random_coords(rng, (n_rows, n_cols), int(rng.integers(0, n_rows * n_cols + 1)))
        pos, crd = to_csr(c, n_rows)
        A = oracle.csr(pos, crd, n_rows, n_cols)
        nnz = int(pos[-1])
        for Q in range(nnz):
            coord, posn, cost = oracle.find_partition([A], Q)
            row = int(np.searchsorted(pos, Q, side="right") - 1)     # pos[row] <= Q < pos[row+1]
            assert coord.tolist() == [row, int(crd[Q])]
            assert posn.tolist() == [[row, Q]] and cost == Q
            # residual after level 0 equals C_j of the listing: x_jp - pos[x_i]
            assert Q - (pos[row] - pos[0]) == posn[0, 1] - pos[row]


def test_spmm_tail_dimension_reading():
    """Loop order i -> j -> k with the dense k innermost: a query that is a
    multiple of N_k lands on k = 0 and on SpMV's boundary; other queries land
    inside the dense loop at k = Q mod N_k (cost scaled by N_k: broadcast rule of
    Section 4.2.2)."""
    rng = np.random.default_rng(3)
    n_rows, n_cols, nk = 11, 13, 8
    c = random_coords(rng, (n_rows, n_cols), 40)
    pos, crd = to_csr(c, n_rows)
    A = oracle.csr(pos, crd, n_rows, n_cols)
    assert oracle.total_cost([A], tail_extent=nk) == 40 * nk
    for Q in range(40 * nk):
        coord, posn, cost = oracle.find_partition([A], Q, tail_extent=nk)
        c1, p1, cost1 = oracle.find_partition([A], Q // nk)
        assert coord[:2].tolist() == c1.tolist() and posn.tolist() == p1.tolist()
        assert coord[2] == Q % nk and cost == Q
    parts = oracle.partition([A], 5, tail_extent=nk,
                             queries=np.array([0, 8 * 3, 8 * 17, 8 * 17, 8 * 39, 320], np.int64))
    assert np.all(parts["coord"][:, 2] == 0)
    assert parts["posn"][:, 0, 1].tolist() == [0, 3, 17, 17, 39, 40]


# --------------------------------------------------------------------------- #
# three vectors against numpy's sort and searchsorted (the case Section 4.2.3 specialises)
# --------------------------------------------------------------------------- #
def test_three_vectors_against_numpy_sort():
    """The boundary of query q is the q-th smallest of all stored indices (numpy.sort of their
    concatenation); every vector's position is numpy.searchsorted of that index; the cost is their sum."""
    rng = np.random.default_rng(11)
    for trial in range(60):
        n = int(rng.integers(1, 200))
        vecs = [to_vector(random_coords(rng, (n,), int(rng.integers(0, n + 1)))) for _ in range(3)]
        ops = [oracle.vector(v, n) for v in vecs]
        everything = np.sort(np.concatenate(vecs))
        for q in range(everything.shape[0]):
            x = int(everything[q])
            at = [int(np.searchsorted(v, x, side="left")) for v in vecs]
            coord, posn, cost = oracle.find_partition(ops, q)
            assert int(coord[0]) == x and posn[:, 0].tolist() == at and cost == sum(at)


# --------------------------------------------------------------------------- #
# properties required of cost functions (Section 3.1), by enumeration
# --------------------------------------------------------------------------- #
def test_cost_is_monotone_and_hierarchically_consistent():
    """C(x) returned with a boundary equals the count of stored entries before
    x; enumerating all coordinates checks monotonicity along the lexicographic
    order and C_m(x+1|.) = C_m(x|.) + C_{m+1}(N|., x) through the total cost
    C(x0..xm+1, 0..) - C(x0..xm, 0..) = entries with that prefix."""
    rng = np.random.default_rng(21)
    shape = (5, 6)
    lists = [random_coords(rng, shape, 11), random_coords(rng, shape, 8)]
    merged = merged_sorted(lists)

    def C(x):                                        # entries strictly before x
        return sum(1 for c in merged if c < tuple(x))

    prev = -1
    for i in range(shape[0]):
        row_total = sum(1 for c in merged if c[0] == i)
        assert C((i + 1, 0)) == C((i, 0)) + row_total            # hierarchical consistency
        for j in range(shape[1] + 1):
            assert C((i, j)) >= prev                              # monotone in lexicographic order
            prev = C((i, j))
    ops = [oracle.dcsr(*to_dcsr(c), *shape) for c in lists]
    for Q in range(len(merged)):
        coord, _, cost = oracle.find_partition(ops, Q)
        assert cost == C(coord.tolist())


def test_coo_boundaries_equal_dcsr_boundaries():
    """A coordinate list and the DCSR form of the same matrices: same boundary coordinates, same
    positions of the non-zeros, same costs (only the row-level positions mean different things:
    stored rows before the boundary row vs non-zeros before it)."""
    rng = np.random.default_rng(321)
    shape = (60, 45)
    for trial in range(10):
        k = int(rng.integers(1, 5))
        cs = [random_coords(rng, shape, int(rng.integers(0, 900))) for _ in range(k)]
        coo = [_make("coo", c, shape) for c in cs]
        dcsr = [_make("dcsr", c, shape) for c in cs]
        for P in (1, 3, 16, 250):
            a, b = oracle.partition(coo, P), oracle.partition(dcsr, P)
            assert np.array_equal(a["coord"], b["coord"])
            assert np.array_equal(a["cost"], b["cost"])
            assert np.array_equal(a["posn"][:, :, 1], b["posn"][:, :, 1])
            for t, c in enumerate(cs):
                starts = np.searchsorted(c[:, 0], a["coord"][:, 0], side="left")
                assert np.array_equal(a["posn"][:, t, 0], starts)


def test_fig3a_as_coordinate_lists(golden_dir):
    g = _load(golden_dir, "fig3a_dcsr_add_partition.json")
    ops = [oracle.coo([c[0] for c in g[key]], [c[1] for c in g[key]], g["n_rows"], g["n_cols"]) for key in ("A", "B")]
    parts = oracle.partition(ops, g["P"])
    assert np.diff(parts["cost"]).tolist() == [6, 6, 6, 6]
    for t, key in enumerate(("A_membership", "B_membership")):
        counts = np.bincount(g[key], minlength=g["P"])
        assert parts["posn"][:, t, 1].tolist() == [0] + np.cumsum(counts).tolist()
    assert parts["coord"][1:-1].tolist() == [[0, 5], [2, 6], [3, 4]]
