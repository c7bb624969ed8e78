"""GPU parity of the row-aware cost variant (nacho_partition_rowcost, nacho_spmv_rowcost) against the
oracle: boundaries bit-exact (coordinates, positions, costs), y within 1e-12 / 1e-5 of the plain sum."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_17198_amd import binding as nb
from paper_2604_17198_amd import workloads
from gpu_util import csr_operand, dev
from util import random_coords, to_csr, tol_ok

pytestmark = pytest.mark.gpu


def _compare(A, P, rc, tag):
    print(f"rowcost partition {tag} rows={A['n_rows']} nnz={int(A['pos'][-1])} P={P} rc={rc}", flush=True)
    got = nb.nacho_partition_rowcost(csr_operand(A), P, rc)
    torch.cuda.synchronize()
    ref = oracle.partition_rowcost([oracle.csr(A["pos"], A["crd"], A["n_rows"], A["n_cols"])], P, rc)
    assert np.array_equal(got["cost"].cpu().numpy(), ref["cost"]), tag
    assert np.array_equal(got["coord"].cpu().numpy().astype(np.int64), ref["coord"]), tag
    assert np.array_equal(got["posn"].cpu().numpy().astype(np.int64), ref["posn"]), tag
    return ref


def _matrix(rng, n_rows, n_cols, nnz, dtype=np.float64):
    c = random_coords(rng, (n_rows, n_cols), nnz)
    pos, crd = to_csr(c, n_rows)
    return {"n_rows": n_rows, "n_cols": n_cols, "pos": pos, "crd": crd,
            "val": rng.uniform(-1, 1, crd.shape[0]).astype(dtype)}


@pytest.mark.parametrize("rc", [1, 3])
def test_partition_random(rc):
    rng = np.random.default_rng(31 + rc)
    for trial in range(8):
        n_rows, n_cols = int(rng.integers(1, 2000)), int(rng.integers(1, 50))      # few columns: column 0 is common
        A = _matrix(rng, n_rows, n_cols, int(rng.integers(0, min(n_rows * n_cols, 15000) + 1)))
        total = int(A["pos"][-1]) + rc * n_rows
        for P in (1, 2, 13, 257, total + 3):
            _compare(A, P, rc, f"random{trial}")


def test_partition_empty_rows_and_heavy_rows():
    rng = np.random.default_rng(41)
    n_rows, n_cols = 50_000, 3000
    lens = {5: 2500, 6: 1, 20_000: 3000, 20_001: 0, 49_999: 700}
    rows = np.repeat(list(lens), list(lens.values()))
    cols = np.concatenate([np.sort(rng.choice(n_cols, l, replace=False)) for l in lens.values()])
    pos, crd = to_csr(np.stack([rows, cols], 1), n_rows)
    A = {"n_rows": n_rows, "n_cols": n_cols, "pos": pos, "crd": crd,
         "val": rng.uniform(-1, 1, crd.shape[0])}
    for rc in (1, 2):
        for P in (3, 64, 1000):
            _compare(A, P, rc, "mostly empty")


def test_config2_scaled_partition_and_balance():
    cfg = workloads.config(2, scale=0.05)
    A = cfg["A"]
    P = nb.rowcost_partitions(csr_operand(A), nb.F64, 1)
    ref = _compare(A, P, 1, "config2@0.05")
    work = np.diff(ref["cost"])
    assert work.max() <= 512 and work.max() - work.min() <= 3


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_spmv_rowcost_values(dtype):
    rng = np.random.default_rng(51)
    tol = 1e-12 if dtype == np.float64 else 1e-5
    cases = [_matrix(rng, 3000, 2500, 20000, dtype), _matrix(rng, 1, 4000, 3000, dtype),
             _matrix(rng, 5000, 3, 9000, dtype)]
    cfg = workloads.config(2, scale=0.02)
    cases.append(dict(cfg["A"], val=cfg["A"]["val"].astype(dtype)))
    for n, A in enumerate(cases):
        x = rng.uniform(-1, 1, A["n_cols"]).astype(dtype)
        ref, s = oracle.spmv(A["pos"], A["crd"], A["val"], x)
        for rc in (1, 4):
            for P in (0, 1, 9, 500):
                print(f"rowcost spmv case{n} rc={rc} P={P} dtype={dtype.__name__}", flush=True)
                y = torch.full((A["n_rows"],), float("nan"), dtype=dev(x).dtype, device="cuda")
                nb.nacho_spmv_rowcost(csr_operand(A), dev(x), y, rc, P=P)
                torch.cuda.synchronize()
                got = y.cpu().numpy()
                assert not np.isnan(got).any()
                assert tol_ok(got, ref, s, tol).all(), (n, rc, P)
                assert np.all(got[np.diff(A["pos"]) == 0] == 0.0)
