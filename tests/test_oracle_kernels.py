"""Pins for the oracle's kernels (no GPU): SpMV, SpMM and k-way union addition
against brute-force dense evaluation on tiny inputs, numpy set routines for the
index sets, and scipy.sparse as a second opinion on medium inputs."""
import json
import os

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from paper_2604_17198_amd import workloads
from util import random_coords, to_csr, to_dcsr, to_vector


def _dense_from(coords, vals, shape):
    D = np.zeros(shape, dtype=np.float64)
    D[tuple(coords.T)] = vals
    return D


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_spmv_spmm_vs_dense(dtype):
    rng = np.random.default_rng(31)
    for trial in range(25):
        n_rows, n_cols = int(rng.integers(1, 25)), int(rng.integers(1, 25))
        c = random_coords(rng, (n_rows, n_cols), int(rng.integers(0, n_rows * n_cols + 1)))
        val = rng.uniform(-1, 1, c.shape[0]).astype(dtype)
        x = rng.uniform(-1, 1, n_cols).astype(dtype)
        pos, crd = to_csr(c, n_rows)
        D = _dense_from(c, val.astype(np.float64), (n_rows, n_cols))
        y, s = oracle.spmv(pos, crd, val, x)
        assert np.allclose(y, D @ x.astype(np.float64), rtol=1e-14, atol=1e-15)
        assert np.allclose(s, np.abs(D) @ np.abs(x.astype(np.float64)), rtol=1e-14, atol=1e-15)
        empty = np.diff(pos) == 0
        assert np.all(y[empty] == 0.0)
        nk = int(rng.integers(1, 9))
        B = rng.uniform(-1, 1, (n_cols, nk)).astype(dtype)
        Cm, S = oracle.spmm(pos, crd, val, B)
        assert np.allclose(Cm, D @ B.astype(np.float64), rtol=1e-14, atol=1e-15)
        assert np.allclose(S, np.abs(D) @ np.abs(B.astype(np.float64)), rtol=1e-14, atol=1e-15)


def test_spmv_is_not_transposed_and_respects_row_order():
    """A non-symmetric hand case: y = A x with A = [[0,2,0],[3,0,4]]."""
    pos = np.array([0, 1, 3], np.int32)
    crd = np.array([1, 0, 2], np.int32)
    val = np.array([2.0, 3.0, 4.0])
    x = np.array([1.0, 10.0, 100.0])
    y, s = oracle.spmv(pos, crd, val, x)
    assert y.tolist() == [20.0, 403.0] and s.tolist() == [20.0, 403.0]
    Cm, _ = oracle.spmm(pos, crd, val, np.stack([x, -x], axis=1))
    assert Cm.tolist() == [[20.0, -20.0], [403.0, -403.0]]


def test_spmv_vs_scipy_on_config1():
    cfg = workloads.config(1)
    A, x = cfg["A"], cfg["x"]
    y, s = oracle.spmv(A["pos"], A["crd"], A["val"], x)
    M = sp.csr_matrix((A["val"], A["crd"], A["pos"]), shape=(A["n_rows"], A["n_cols"]))
    ref = M @ x
    assert np.all(np.abs(y - ref) <= 1e-13 * np.maximum(np.abs(ref), s) + 1e-300)
    assert np.all(y[np.diff(A["pos"]) == 0] == 0.0)


def test_union_of_fig1_vectors(golden_dir):
    with open(os.path.join(golden_dir, "fig1_three_vectors.json")) as f:
        g = json.load(f)
    idx = [np.array(g[n], np.int32) for n in "abc"]
    vals = [np.arange(1, len(i) + 1, dtype=np.float64) * 10 ** t for t, i in enumerate(idx)]
    oi, ov, oa = oracle.spadd_vec(idx, vals)
    ref = np.union1d(np.union1d(idx[0], idx[1]), idx[2])
    assert oi.tolist() == ref.tolist() == [1, 2, 4, 5, 9, 10, 11]
    # 1: a0+b0+c0 ; 9: a2+b3+c2
    assert ov[0] == 1 + 10 + 100 and ov[4] == 3 + 40 + 300 and ov[1] == 20


@pytest.mark.parametrize("k", [1, 2, 3, 6])
def test_spadd_vec_vs_dense(k):
    rng = np.random.default_rng(41 + k)
    for trial in range(30):
        n = int(rng.integers(1, 120))
        idx, vals, dense, mask = [], [], np.zeros(n), np.zeros(n, bool)
        dabs = np.zeros(n)
        for t in range(k):
            c = to_vector(random_coords(rng, (n,), int(rng.integers(0, n + 1))))
            if trial % 5 == 0 and t > 0:
                c = idx[0].copy()
            v = rng.uniform(-1, 1, c.shape[0]).astype(np.float32)
            idx.append(c)
            vals.append(v)
            dense[c] += v.astype(np.float64)
            dabs[c] += np.abs(v.astype(np.float64))
            mask[c] = True
        oi, ov, oa = oracle.spadd_vec(idx, vals)
        assert oi.tolist() == np.flatnonzero(mask).tolist()          # structural union, sorted
        assert np.allclose(ov, dense[mask], rtol=1e-15, atol=1e-16)
        assert np.allclose(oa, dabs[mask], rtol=1e-15, atol=1e-16)


@pytest.mark.parametrize("k", [1, 2, 3])
def test_spadd_dcsr_and_csr_vs_dense(k):
    rng = np.random.default_rng(51 + k)
    for trial in range(30):
        shape = (int(rng.integers(1, 14)), int(rng.integers(1, 14)))
        mats_d, mats_c = [], []
        dense, mask = np.zeros(shape), np.zeros(shape, bool)
        for t in range(k):
            c = random_coords(rng, shape, int(rng.integers(0, shape[0] * shape[1] + 1)))
            v = rng.uniform(-1, 1, c.shape[0]).astype(np.float32)
            p0, c0, p1, c1 = to_dcsr(c)
            mats_d.append({"pos0": p0, "crd0": c0, "pos1": p1, "crd1": c1, "val": v})
            pos, crd = to_csr(c, shape[0])
            mats_c.append({"pos": pos, "crd": crd, "val": v})
            dense[tuple(c.T)] += v.astype(np.float64)
            mask[tuple(c.T)] = True
        out = oracle.spadd_dcsr(mats_d)
        rows = np.flatnonzero(mask.any(axis=1))
        assert out["crd0"].tolist() == rows.tolist() and out["pos0"].tolist() == [0, rows.shape[0]]
        assert out["pos1"].tolist() == [0] + np.cumsum(mask.sum(axis=1)[rows]).tolist()
        rr, cc = np.nonzero(mask)                                     # row-major = lexicographic
        assert out["crd1"].tolist() == cc.tolist()
        assert np.allclose(out["val"], dense[rr, cc], rtol=1e-15, atol=1e-16)
        outc = oracle.spadd_csr(mats_c)
        assert outc["pos"].tolist() == [0] + np.cumsum(mask.sum(axis=1)).tolist()
        assert outc["crd"].tolist() == cc.tolist()
        assert np.allclose(outc["val"], dense[rr, cc], rtol=1e-15, atol=1e-16)


def test_spadd_dcsr_vs_scipy_medium():
    cfg = workloads.config(4, scale=0.002)
    A, B = cfg["ops"]
    out = oracle.spadd_dcsr([A, B])

    def to_sp(M):
        rows = np.repeat(M["crd0"], np.diff(M["pos1"]))
        return sp.csr_matrix((M["val"].astype(np.float64), (rows, M["crd1"])),
                             shape=(cfg["n_rows"], cfg["n_cols"]))

    ref = (to_sp(A) + to_sp(B)).tocsr()
    ref.sort_indices()
    ref_rows = np.flatnonzero(np.diff(ref.indptr))
    assert out["crd0"].tolist() == ref_rows.tolist()
    assert out["crd1"].tolist() == ref.indices.tolist()
    assert np.allclose(out["val"], ref.data, rtol=1e-14, atol=1e-16)
    assert out["pos1"].tolist() == ref.indptr[np.append(ref_rows, ref_rows[-1] + 1)].tolist()


def test_workload_recipe_matches_its_specification():
    """Configuration 1: 4096 rows, ~40k nnz, 30 % empty rows, a few rows of
    thousands of entries, sorted unique columns."""
    A = workloads.config(1)["A"]
    d = np.diff(A["pos"])
    assert A["n_rows"] == 4096 and abs(int(A["pos"][-1]) - 40_000) < 400
    assert abs((d == 0).mean() - 0.30) < 0.01 and np.sort(d)[-3:].min() >= 1000
    for r in np.flatnonzero(d > 1)[:200]:
        seg = A["crd"][A["pos"][r]:A["pos"][r + 1]]
        assert np.all(np.diff(seg) > 0)
    c3 = workloads.config(3, scale=0.001)
    a, b, c = (o["i"] for o in c3["ops"])
    assert np.all(np.diff(a) > 0) and np.all(np.diff(b) > 0) and np.all(np.diff(c) > 0)
    assert 0.18 < np.isin(b, a).mean() < 0.25


def test_intersection_of_fig1_vectors(golden_dir):
    """The three-finger listing of Section 2.1 on the vectors of Figure 1: only
    coordinates 1 and 9 are stored by all of a, b and c."""
    with open(os.path.join(golden_dir, "fig1_three_vectors.json")) as f:
        g = json.load(f)
    idx = [np.array(g[n], np.int32) for n in "abc"]
    vals = [np.arange(2, len(i) + 2, dtype=np.float64) * (t + 1) for t, i in enumerate(idx)]
    oi, ov, oa = oracle.spmul_vec(idx, vals)
    assert oi.tolist() == [1, 9]
    # 1: a0*b0*c0 ; 9: a2*b3*c2
    assert ov.tolist() == [2 * 4 * 6, 4 * 10 * 12] and oa.tolist() == ov.tolist()


@pytest.mark.parametrize("k", [1, 2, 3, 5])
def test_spmul_vec_and_csr_vs_dense(k):
    rng = np.random.default_rng(71 + k)
    for trial in range(40):
        shape = (int(rng.integers(1, 12)), int(rng.integers(1, 30)))
        mats, vec_i, vec_v = [], [], []
        dense = np.ones(shape)
        mask = np.ones(shape, bool)
        for t in range(k):
            nmax = shape[0] * shape[1]
            c = random_coords(rng, shape, int(rng.integers(nmax // 2, nmax + 1)))
            if trial % 7 == 0 and t > 0:
                c = random_coords(rng, shape, 0)                      # an empty operand: empty result
            v = rng.uniform(-1, 1, c.shape[0]).astype(np.float64)
            pos, crd = to_csr(c, shape[0])
            mats.append({"pos": pos, "crd": crd, "val": v})
            m = np.zeros(shape, bool)
            m[tuple(c.T)] = True
            d = np.zeros(shape)
            d[tuple(c.T)] = v
            mask &= m
            dense *= d
            # the same data as one long sparse vector (row-major linear index)
            vec_i.append((c[:, 0] * shape[1] + c[:, 1]).astype(np.int32))
            vec_v.append(v)
        out = oracle.spmul_csr(mats)
        rr, cc = np.nonzero(mask)
        assert out["pos"].tolist() == [0] + np.cumsum(mask.sum(axis=1)).tolist()
        assert out["crd"].tolist() == cc.tolist()
        assert np.allclose(out["val"], dense[rr, cc], rtol=1e-14, atol=0)
        oi, ov, _ = oracle.spmul_vec(vec_i, vec_v)
        ref = vec_i[0]
        for t in range(1, k):
            ref = np.intersect1d(ref, vec_i[t])
        assert oi.tolist() == ref.tolist() == (rr * shape[1] + cc).tolist()
        assert np.allclose(ov, dense[rr, cc], rtol=1e-14, atol=0)


def test_spmul_csr_vs_scipy_medium():
    cfg = workloads.csr_add_config(2, n=3000, nnz_each=200_000)
    A, B = cfg["ops"]
    out = oracle.spmul_csr([A, B])

    def to_sp(M):
        return sp.csr_matrix((M["val"].astype(np.float64), M["crd"], M["pos"]), shape=(cfg["n_rows"], cfg["n_cols"]))

    ref = to_sp(A).multiply(to_sp(B)).tocsr()
    ref.sort_indices()
    assert out["pos"].tolist() == ref.indptr.tolist() and out["crd"].tolist() == ref.indices.tolist()
    assert np.allclose(out["val"], ref.data, rtol=1e-14, atol=0) and out["crd"].shape[0] > 1000


@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_coo_add_and_multiply_vs_dense_and_scipy(k):
    rng = np.random.default_rng(40 + k)
    shape = (31, 23)
    for trial in range(10):
        mats, dense_sum, dense_prod = [], np.zeros(shape), np.ones(shape)
        any_mask, all_mask = np.zeros(shape, bool), np.ones(shape, bool)
        sp_sum = sp.csr_matrix(shape)
        for t in range(k):
            c = random_coords(rng, shape, int(rng.integers(0, 400)))
            v = rng.uniform(0.5, 1.5, c.shape[0]) * rng.choice([-1, 1], c.shape[0])
            mats.append({"row": c[:, 0].astype(np.int32), "col": c[:, 1].astype(np.int32), "val": v})
            d = np.zeros(shape)
            d[c[:, 0], c[:, 1]] = v
            m = np.zeros(shape, bool)
            m[c[:, 0], c[:, 1]] = True
            dense_sum += d
            dense_prod *= d
            any_mask |= m
            all_mask &= m
            sp_sum = sp_sum + sp.csr_matrix((v, (c[:, 0], c[:, 1])), shape=shape)
        z = oracle.spadd_coo(mats)
        ii, jj = np.nonzero(any_mask)                     # row-major order = sorted by (row, col)
        assert z["row"].tolist() == ii.tolist() and z["col"].tolist() == jj.tolist()
        np.testing.assert_allclose(z["val"], dense_sum[ii, jj], rtol=1e-12, atol=1e-15)
        zs = sp_sum.tocoo()
        np.testing.assert_allclose(sp.csr_matrix((z["val"], (z["row"], z["col"])), shape=shape).toarray(),
                                   zs.toarray(), rtol=1e-12, atol=1e-15)
        y = oracle.spmul_coo(mats)
        ii, jj = np.nonzero(all_mask)
        assert y["row"].tolist() == ii.tolist() and y["col"].tolist() == jj.tolist()
        np.testing.assert_allclose(y["val"], dense_prod[ii, jj], rtol=1e-12)


def test_coo_results_equal_dcsr_results():
    rng = np.random.default_rng(44)
    shape = (200, 150)
    cs = [random_coords(rng, shape, 6000) for _ in range(3)]
    vs = [rng.standard_normal(c.shape[0]) for c in cs]
    coo = [{"row": c[:, 0].astype(np.int32), "col": c[:, 1].astype(np.int32), "val": v} for c, v in zip(cs, vs)]
    dc = []
    for c, v in zip(cs, vs):
        p0, c0, p1, c1 = to_dcsr(c)
        dc.append({"pos0": p0, "crd0": c0, "pos1": p1, "crd1": c1, "val": v})
    for f_coo, f_dcsr in ((oracle.spadd_coo, oracle.spadd_dcsr), (oracle.spmul_coo, oracle.spmul_dcsr)):
        a, b = f_coo(coo), f_dcsr(dc)
        assert np.array_equal(a["col"], b["crd1"]) and np.array_equal(a["val"], b["val"])
        assert np.array_equal(a["row"], np.repeat(b["crd0"], np.diff(b["pos1"])))
