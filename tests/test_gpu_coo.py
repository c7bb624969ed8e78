"""GPU parity for coordinate-list (COO) operands: nacho_partition, nacho_spadd_k and
nacho_spmul_k vs the oracle.  Boundaries and index arrays bit-exact; values within
1e-5 (fp32) / 1e-12 (fp64) of max(|ref|, sum |terms|)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_17198_amd import binding as nb
from paper_2604_17198_amd import workloads
from gpu_util import dev, parts_to_numpy
from util import random_coords, tol_ok

pytestmark = pytest.mark.gpu

TOL = {np.float32: 1e-5, np.float64: 1e-12}


def _ops(cs, shape, vals=None):
    g, o = [], []
    for t, c in enumerate(cs):
        r, cc = c[:, 0].astype(np.int32), c[:, 1].astype(np.int32)
        g.append(nb.coo(dev(r), dev(cc), shape[0], shape[1], None if vals is None else dev(vals[t])))
        o.append(oracle.coo(r, cc, shape[0], shape[1]))
    return g, o


def _compare_parts(got, ref, tag):
    assert np.array_equal(got["cost"], ref["cost"]), tag
    assert np.array_equal(got["coord"].astype(np.int64), ref["coord"]), tag
    assert np.array_equal(got["posn"].astype(np.int64), ref["posn"]), tag


@pytest.mark.parametrize("k", [1, 2, 3, 4, 8])
def test_partition_random(k):
    rng = np.random.default_rng(300 + k)
    for trial in range(6):
        shape = [(1, 50), (50, 1), (40, 60), (3000, 2000), (2**20, 2**20), (7, 100000)][trial]
        cs = []
        for t in range(k):
            n = int(rng.integers(0, 4000))
            if shape[0] * shape[1] < 10**7:
                c = random_coords(rng, shape, n)
            else:
                key = np.unique(rng.integers(0, shape[0], n).astype(np.int64) * shape[1] + rng.integers(0, shape[1], n))
                c = np.stack([key // shape[1], key % shape[1]], axis=1)
            if trial == 2 and t > 0:
                c = cs[0].copy()                       # every pair tied across operands
            cs.append(c)
        g, o = _ops(cs, shape)
        total = sum(len(c) for c in cs)
        for P in (1, 2, 7, 64, 300, total + 2):
            print(f"partition coo k={k} trial={trial} shape={shape} total={total} P={P}", flush=True)
            got = parts_to_numpy(nb.nacho_partition(g, P))
            _compare_parts(got, oracle.partition(o, P), (k, trial, P))


def test_partition_long_rows_and_many_duplicated_rows():
    """Row coordinates repeat thousands of times (one long row) and boundaries fall inside rows."""
    rng = np.random.default_rng(5)
    shape = (50, 200000)
    cs = []
    for t in range(3):
        rows = np.sort(rng.choice([3, 3, 3, 17, 40], 30000))
        key = np.unique(rows.astype(np.int64) * shape[1] + rng.integers(0, shape[1], 30000))
        cs.append(np.stack([key // shape[1], key % shape[1]], axis=1))
    g, o = _ops(cs, shape)
    for P in (5, 1000):
        got = parts_to_numpy(nb.nacho_partition(g, P))
        _compare_parts(got, oracle.partition(o, P), P)


def _run(fn_gpu, fn_ref, cs, vals, shape, P, tag, cap=None):
    k = len(cs)
    dtype = vals[0].dtype.type
    print(f"coo {tag} k={k} shape={shape} nnz={[len(c) for c in cs]} P={P} {dtype.__name__}", flush=True)
    g, _ = _ops(cs, shape, vals)
    tdt = torch.float32 if dtype == np.float32 else torch.float64
    full = sum(len(c) for c in cs)
    out = nb.SparseOut("coo", 0, full if cap is None else cap, tdt, "cuda")
    fn_gpu(g, out, P=P)
    torch.cuda.synchronize()
    nnz = int(out.counts.cpu().numpy()[1])
    status = int(out.status.cpu().numpy()[0])
    ref = fn_ref([{"row": c[:, 0].astype(np.int32), "col": c[:, 1].astype(np.int32), "val": v}
                  for c, v in zip(cs, vals)])
    return out, nnz, status, ref


def _check(fn_gpu, fn_ref, cs, vals, shape, P, tag):
    out, nnz, status, ref = _run(fn_gpu, fn_ref, cs, vals, shape, P, tag)
    dtype = vals[0].dtype.type
    assert status == 0 and nnz == ref["row"].shape[0], (tag, status, nnz, ref["row"].shape[0])
    assert np.array_equal(out.crd0.cpu().numpy()[:nnz], ref["row"]), tag
    assert np.array_equal(out.crd1.cpu().numpy()[:nnz], ref["col"]), tag
    assert out.pos1.cpu().numpy().tolist() == [0, nnz], tag
    ok = tol_ok(out.val.cpu().numpy()[:nnz], ref["val"], ref["abs"], TOL[dtype])
    assert ok.all(), (tag, int((~ok).sum()))


@pytest.mark.parametrize("k", [1, 2, 3, 4, 8])
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_add_and_multiply_random(k, dtype):
    rng = np.random.default_rng(600 + k)
    for trial in range(5):
        shape = [(30, 40), (500, 300), (64, 5000), (2000, 2000), (9, 9)][trial]
        dens = [0.5, 0.2, 0.1, 0.01, 0.95][trial]
        cs, vals = [], []
        for t in range(k):
            c = random_coords(rng, shape, int(dens * shape[0] * shape[1] * rng.uniform(0.3, 1.0)))
            if trial == 4 and t == k - 1 and k > 1:
                c = np.zeros((0, 2), np.int64)           # an empty operand
            cs.append(c)
            vals.append((rng.uniform(0.5, 1.5, c.shape[0]) * rng.choice([-1, 1], c.shape[0])).astype(dtype))
        for P in (0, 1, 9, 400):
            _check(nb.nacho_spadd_k, oracle.spadd_coo, cs, vals, shape, P, f"add{trial}")
            _check(nb.nacho_spmul_k, oracle.spmul_coo, cs, vals, shape, P, f"mul{trial}")


def test_capacity_overflow_is_reported():
    rng = np.random.default_rng(2)
    shape = (300, 300)
    cs = [random_coords(rng, shape, 20000) for _ in range(2)]
    vals = [np.ones(len(c), np.float32) for c in cs]
    out, nnz, status, ref = _run(nb.nacho_spadd_k, oracle.spadd_coo, cs, vals, shape, 0, "cap",
                                 cap=10000)
    assert status == -4 and nnz == ref["row"].shape[0]
    assert np.array_equal(out.crd0.cpu().numpy()[:10000], ref["row"][:10000])


def test_config4_matrices_as_coordinate_lists():
    """The two matrices of configuration 4 (1M x 1M, ~20M non-zeros each) stored as coordinate
    lists: COO + COO and the COO Hadamard product at full size."""
    cfg = workloads.config(4)
    cs, vals = [], []
    for m in cfg["ops"]:
        rows = np.repeat(m["crd0"], np.diff(m["pos1"]))
        cs.append(np.stack([rows, m["crd1"]], axis=1))
        vals.append(m["val"])
    shape = (cfg["n_rows"], cfg["n_cols"])
    _check(nb.nacho_spadd_k, oracle.spadd_coo, cs, vals, shape, 0, "config4 add")
    _check(nb.nacho_spmul_k, oracle.spmul_coo, cs, vals, shape, 0, "config4 mul")
    g, o = _ops(cs, shape)
    got = parts_to_numpy(nb.nacho_partition(g, 5000))
    _compare_parts(got, oracle.partition(o, 5000), "config4 partition")
