"""Pins of the oracle's nested-intersection functions (Section 3.3): the DCSR
Hadamard product, the remapped cost function and Algorithm 2, against the
paper's figures, brute force from the definitions, scipy and invariants."""
import json
import os

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from util import random_coords, to_dcsr


def _load(golden_dir, name):
    with open(os.path.join(golden_dir, name)) as f:
        return json.load(f)


def _mat(coords, vals=None):
    coords = np.asarray(coords, dtype=np.int64).reshape(-1, 2)
    p0, c0, p1, c1 = to_dcsr(coords)
    if vals is None:
        vals = np.ones(coords.shape[0])
    return {"pos0": p0, "crd0": c0, "pos1": p1, "crd1": c1, "val": np.asarray(vals, dtype=np.float64)}


def _entries_of(m):
    """(row, col) of every stored entry in storage order."""
    rows = np.repeat(m["crd0"], np.diff(m["pos1"]))
    return list(zip(rows.tolist(), m["crd1"].tolist()))


# --------------------------------------------------------------------------- #
# the paper's worked examples
# --------------------------------------------------------------------------- #
def test_fig5_remapped_cost_function(golden_dir):
    g = _load(golden_dir, "fig5_remapped_cost.json")
    A, B = _mat(g["A"]), _mat(g["B"])
    r = oracle.recursive_partition_dcsr([A, B], g["n_cols"], 2)
    assert r["rows"].tolist() == g["intersected_rows"]
    assert r["T"].tolist() == g["T"]
    assert r["Tprime"].tolist() == g["Tprime"]
    # the remapped trees of the figure: row i' of an operand is its row rows[i']
    for m, key in ((A, "remapped_A"), (B, "remapped_B")):
        remap = {int(i): n for n, i in enumerate(r["rows"])}
        got = [[remap[i], j] for i, j in _entries_of(m) if i in remap]
        assert got == g[key]


def test_fig3b_dcsr_multiplication(golden_dir):
    g = _load(golden_dir, "fig3b_dcsr_mul_partition.json")
    A, B = _mat(g["A"]), _mat(g["B"])
    P = g["P"]
    r = oracle.recursive_partition_dcsr([A, B], g["n_cols"], P)
    skipped = set(range(g["n_rows"])) - set(r["rows"].tolist())
    assert sorted(skipped) == g["skipped_rows"]
    assert np.diff(r["cost"]).tolist() == [4, 4, 4, 4]
    # colours -> entries of each operand in each chunk; gray entries are in no chunk
    for t, (m, key) in enumerate(((A, "A_membership"), (B, "B_membership"))):
        memb = np.array(g[key])
        counts = np.bincount(memb[memb >= 0], minlength=P)
        assert r["before"][:, t].tolist() == [0] + np.cumsum(counts).tolist()
        # membership of every stored entry from the boundaries' positions in crd1
        ent = _entries_of(m)
        inter = set(r["rows"].tolist())
        got = []
        for q, (i, j) in enumerate(ent):
            if i not in inter:
                got.append(-1)
                continue
            got.append(int(np.searchsorted(r["lpos"][1:, t], q, side="right")))
        assert got == memb.tolist()
    cuts = [[int(r["rows"][c[0]]), int(c[1])] for c in r["coord"][1:-1]]
    drawn = g["drawn_cuts_row_col"]
    assert cuts[0] == drawn[0] and cuts[1] == drawn[1]
    # third cut: drawn at the low end of a flat stretch, the search takes the high end
    assert cuts[2][0] == drawn[2][0] and cuts[2][1] >= drawn[2][1] and cuts[2] == [2, 6]
    stored = {tuple(c) for c in g["A"]} | {tuple(c) for c in g["B"]}
    assert all((2, j) not in stored for j in range(drawn[2][1], cuts[2][1]))
    # and the product itself (pattern read off the figure)
    z = oracle.spmul_dcsr([A, B])
    assert _entries_of(z) == [(0, 0), (0, 3), (0, 4), (2, 6), (2, 7)]


# --------------------------------------------------------------------------- #
# Hadamard product against definitions and scipy
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_spmul_dcsr_vs_dense(k):
    rng = np.random.default_rng(100 + k)
    shape = (23, 17)
    for trial in range(20):
        mats, dense = [], np.ones(shape)
        stored = np.ones(shape, dtype=bool)
        for t in range(k):
            c = random_coords(rng, shape, int(rng.integers(0, 200)))
            v = rng.standard_normal(c.shape[0])
            mats.append(_mat(c, v))
            d = np.zeros(shape)
            d[c[:, 0], c[:, 1]] = v
            m = np.zeros(shape, dtype=bool)
            m[c[:, 0], c[:, 1]] = True
            dense *= d
            stored &= m
        z = oracle.spmul_dcsr(mats)
        ii, jj = np.nonzero(stored)
        assert _entries_of(z) == list(zip(ii.tolist(), jj.tolist()))
        np.testing.assert_allclose(z["val"], dense[ii, jj], rtol=1e-13, atol=0)
        # stored rows are exactly the rows with an entry; pos1 is their running count
        assert z["crd0"].tolist() == sorted(set(ii.tolist()))
        assert z["pos0"].tolist() == [0, z["crd0"].shape[0]]
        assert z["pos1"].tolist() == [0] + np.cumsum(np.bincount(ii, minlength=shape[0])[z["crd0"]]).tolist()


def test_spmul_dcsr_vs_scipy_medium():
    rng = np.random.default_rng(77)
    shape = (3000, 2000)

    def rand():
        # a third of the rows empty, different per operand, so rows are really skipped
        c = random_coords(rng, shape, 60000)
        keep = rng.random(shape[0]) > 0.35
        c = c[keep[c[:, 0]]]
        return c, rng.standard_normal(c.shape[0])

    (ca, va), (cb, vb) = rand(), rand()
    z = oracle.spmul_dcsr([_mat(ca, va), _mat(cb, vb)])
    SA = sp.csr_matrix((va, (ca[:, 0], ca[:, 1])), shape=shape)
    SB = sp.csr_matrix((vb, (cb[:, 0], cb[:, 1])), shape=shape)
    # scipy drops nothing by pattern when both store the entry and the values are non-zero
    ref = SA.multiply(SB).tocsr()
    ref.sort_indices()
    rows = np.repeat(z["crd0"], np.diff(z["pos1"]))
    got = sp.csr_matrix((z["val"], (rows, z["crd1"])), shape=shape)
    got.sort_indices()
    assert np.array_equal(got.indptr, ref.indptr) and np.array_equal(got.indices, ref.indices)
    np.testing.assert_allclose(got.data, ref.data, rtol=1e-13)
    assert z["crd0"].tolist() == np.flatnonzero(np.diff(ref.indptr)).tolist()


# --------------------------------------------------------------------------- #
# Algorithm 2 against brute force written from the definitions
# --------------------------------------------------------------------------- #
def _brute_boundary(coord_lists, inter_rows, n_cols, Q):
    """Highest (i', j) in lexicographic order whose cost (stored entries of all operands in
    intersected rows lexicographically before it) is <= Q, level by level as Algorithm 1
    prescribes, every cost evaluated by counting."""
    M = len(inter_rows)

    def cost_rows(x):       # C'_i(x): entries in the intersected rows i'_0 .. i'_{x-1}
        rows = set(inter_rows[:x])
        return sum(1 for cl in coord_lists for (i, j) in cl if i in rows)

    x = max(xx for xx in range(M + 1) if cost_rows(xx) <= Q)
    R = Q - cost_rows(x)
    if x == M:
        return x, 0, Q - R
    row = inter_rows[x]

    def cost_cols(j):
        return sum(1 for cl in coord_lists for (i, jj) in cl if i == row and jj < j)

    j = max(jj for jj in range(n_cols + 1) if cost_cols(jj) <= R)
    return x, j, Q - (R - cost_cols(j))


@pytest.mark.parametrize("k", [2, 3, 4])
def test_recursive_partition_vs_brute_force(k):
    rng = np.random.default_rng(500 + k)
    shape = (14, 11)
    for trial in range(25):
        lists, mats = [], []
        for t in range(k):
            c = random_coords(rng, shape, int(rng.integers(1, 90)))
            lists.append([(int(a), int(b)) for a, b in c])
            mats.append(_mat(c))
        inter = sorted(set.intersection(*[{i for i, _ in cl} for cl in lists]))
        P = int(rng.integers(1, 9))
        r = oracle.recursive_partition_dcsr(mats, shape[1], P)
        assert r["rows"].tolist() == inter
        total = sum(1 for cl in lists for (i, _) in cl if i in set(inter))
        assert int(r["Tprime"][-1]) == total == int(r["cost"][-1])
        for b in range(1, P):
            Q = b * total // P
            if Q >= total:
                continue
            x, j, c = _brute_boundary(lists, inter, shape[1], Q)
            assert r["coord"][b].tolist() == [x, j]
            assert int(r["cost"][b]) == c
            # tightness (Theorem 1): the boundary's cost misses the query by less than k
            assert 0 <= Q - c < k
            for t in range(k):
                bef = sum(1 for (i, jj) in lists[t]
                          if i in set(inter) and (inter.index(i), jj) < (x, j))
                assert int(r["before"][b, t]) == bef
        assert np.all(np.diff(r["cost"]) >= 0)
        # imbalance of equally spaced queries: at most ideal share + k - 1 ... 2 (k - 1) apart
        if total:
            w = np.diff(r["cost"])
            assert w.max() - w.min() <= 2 * k


def test_partitions_compose_to_the_whole_product():
    """Equal coordinates of different operands fall in the same partition (Section 6), so the
    product restricted to each partition's entries, concatenated, is the whole product."""
    rng = np.random.default_rng(9)
    shape = (40, 30)
    for k in (2, 3):
        cs = [random_coords(rng, shape, 500) for _ in range(k)]
        mats = [_mat(c, rng.standard_normal(c.shape[0])) for c in cs]
        P = 7
        r = oracle.recursive_partition_dcsr(mats, shape[1], P)
        z = oracle.spmul_dcsr(mats)
        whole = dict(zip(_entries_of(z), z["val"].tolist()))
        pieces = {}
        inter = set(r["rows"].tolist())
        for p in range(P):
            per_op = []
            for t, m in enumerate(mats):
                ent = _entries_of(m)
                sel = {}
                # entries of operand t inside the partition: in intersected rows, between the boundaries
                n_before = 0
                for q, (i, j) in enumerate(ent):
                    if i not in inter:
                        continue
                    if r["before"][p, t] <= n_before < r["before"][p + 1, t]:
                        sel[(i, j)] = m["val"][q]
                    n_before += 1
                per_op.append(sel)
            common = set.intersection(*[set(s) for s in per_op])
            for c in common:
                assert c not in pieces
                pieces[c] = float(np.prod([s[c] for s in per_op]))
        assert set(pieces) == set(whole)
        for c in whole:
            assert pieces[c] == pytest.approx(whole[c], rel=1e-13)


def test_degenerate_cases():
    A = _mat([[1, 1], [1, 2], [3, 0]])
    empty = _mat(np.zeros((0, 2), dtype=np.int64))
    for ops in ([A, empty], [empty, empty]):
        z = oracle.spmul_dcsr(ops)
        assert z["pos0"].tolist() == [0, 0] and z["crd1"].shape[0] == 0
        r = oracle.recursive_partition_dcsr(ops, 4, 3)
        assert r["rows"].shape[0] == 0 and r["cost"].tolist() == [0, 0, 0, 0]
    # rows match but no column does: every row of the product is empty and none is stored
    B = _mat([[1, 0], [3, 3]])
    z = oracle.spmul_dcsr([A, B])
    assert z["pos0"].tolist() == [0, 0] and z["pos1"].tolist() == [0]
    r = oracle.recursive_partition_dcsr([A, B], 4, 2)
    assert r["rows"].tolist() == [1, 3] and r["T"].tolist() == [3, 2]
    # one operand: every row intersects, the remapped space is the operand itself
    r = oracle.recursive_partition_dcsr([A], 4, 3)
    ref = oracle.partition([oracle.dcsr(A["pos0"], A["crd0"], A["pos1"], A["crd1"], 5, 4)], 3)
    assert r["before"][:, 0].tolist() == ref["posn"][:, 0, 1].tolist()
