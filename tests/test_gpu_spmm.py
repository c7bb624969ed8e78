"""GPU parity: nacho_spmm vs the oracle (C_ik = sum_j A_ij B_jk in double /
long double).  Tolerance |C - C_ref| <= tol * max(|C_ref|, sum_j |A_ij B_jk|),
tol = 1e-5 (fp32), 1e-12 (fp64); rows of C for empty rows of A are exactly 0."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_17198_amd import binding as nb
from paper_2604_17198_amd import workloads
from gpu_util import csr_operand, dev
from util import random_coords, to_csr, tol_ok

pytestmark = pytest.mark.gpu

TOL = {np.float32: 1e-5, np.float64: 1e-12}


def _check(A, B, P, tag):
    dtype = A["val"].dtype.type
    print(f"spmm {tag} rows={A['n_rows']} nnz={int(A['pos'][-1])} n={B.shape[1]} P={P} {dtype.__name__}", flush=True)
    Bd = dev(B)
    C = torch.full((A["n_rows"], B.shape[1]), float("nan"), dtype=Bd.dtype, device="cuda")
    nb.nacho_spmm(csr_operand(A), Bd, C, P=P)
    torch.cuda.synchronize()
    got = C.cpu().numpy()
    ref, sabs = oracle.spmm(A["pos"], A["crd"], A["val"], B)
    assert not np.isnan(got).any(), f"{tag}: part of C never written"
    ok = tol_ok(got, ref, sabs, TOL[dtype])
    assert ok.all(), (tag, int((~ok).sum()))
    assert np.all(got[np.diff(A["pos"]) == 0] == 0.0)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_random_small(dtype):
    rng = np.random.default_rng(21)
    for trial in range(8):
        n_rows, n_cols = int(rng.integers(1, 2000)), int(rng.integers(1, 2000))
        nnz = int(rng.integers(0, min(n_rows * n_cols, 15000) + 1))
        c = random_coords(rng, (n_rows, n_cols), nnz)
        pos, crd = to_csr(c, n_rows)
        A = {"n_rows": n_rows, "n_cols": n_cols, "pos": pos, "crd": crd,
             "val": rng.uniform(-1, 1, nnz).astype(dtype)}
        n = int(rng.choice([1, 7, 32, 64]))
        B = rng.uniform(-1, 1, (n_cols, n)).astype(dtype)
        for P in (0, 1, 11, nnz + 3):
            _check(A, B, P, f"random{trial}")


def test_degenerate_shapes():
    rng = np.random.default_rng(22)
    cases = {
        "empty": (np.zeros((0, 2), np.int64), (300, 5)),
        "one_row": (np.stack([np.zeros(4000, np.int64), np.arange(4000)], 1), (1, 4000)),
        "heavy_mid": (np.stack([np.full(5000, 777, np.int64), np.arange(5000)], 1), (3000, 5000)),
    }
    for name, (c, shape) in cases.items():
        pos, crd = to_csr(c, shape[0])
        A = {"n_rows": shape[0], "n_cols": shape[1], "pos": pos, "crd": crd,
             "val": rng.uniform(-1, 1, c.shape[0]).astype(np.float32)}
        B = rng.uniform(-1, 1, (shape[1], 64)).astype(np.float32)
        for P in (0, 5):
            _check(A, B, P, name)


def test_long_runs_of_empty_rows():
    rng = np.random.default_rng(23)
    n_rows, n_cols = 300_000, 3000
    lens = {90_000: 2000, 90_001: 1, 90_600: 30, 200_000: 1500, 200_513: 5, 299_999: 300}
    rows = np.repeat(list(lens), list(lens.values()))
    cols = np.concatenate([np.sort(rng.choice(n_cols, l, replace=False)) for l in lens.values()])
    pos, crd = to_csr(np.stack([rows, cols], 1), n_rows)
    A = {"n_rows": n_rows, "n_cols": n_cols, "pos": pos, "crd": crd,
         "val": rng.uniform(-1, 1, crd.shape[0]).astype(np.float32)}
    for n in (64, 9):
        B = rng.uniform(-1, 1, (n_cols, n)).astype(np.float32)
        for P in (0, 1, 6):
            _check(A, B, P, "empty runs")


def test_leading_dimensions():
    rng = np.random.default_rng(23)
    c = random_coords(rng, (500, 400), 6000)
    pos, crd = to_csr(c, 500)
    A = {"n_rows": 500, "n_cols": 400, "pos": pos, "crd": crd, "val": rng.uniform(-1, 1, 6000).astype(np.float32)}
    Bfull = dev(rng.uniform(-1, 1, (400, 80)).astype(np.float32))
    Cfull = torch.zeros((500, 96), dtype=torch.float32, device="cuda")
    B, C = Bfull[:, :48], Cfull[:, :48]
    nb.nacho_spmm(csr_operand(A), B, C)
    torch.cuda.synchronize()
    ref, sabs = oracle.spmm(pos, crd, A["val"], B.cpu().numpy())
    assert tol_ok(C.cpu().numpy(), ref, sabs, 1e-5).all()
    assert torch.all(Cfull[:, 48:] == 0)


def test_config5_scaled():
    cfg = workloads.config(5, scale=0.02)
    _check(cfg["A"], cfg["B"], 0, "config5@0.02")


def test_config5_full_size():
    cfg = workloads.config(5)
    _check(cfg["A"], cfg["B"], 0, "config5 full")


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_more_than_64_dense_columns(dtype):
    """Wider operands go through the executing kernel in stretches of 64 columns (ragged last one)."""
    rng = np.random.default_rng(33)
    cfg = workloads.config(5, scale=0.01)
    A = dict(cfg["A"])
    A["val"] = A["val"].astype(dtype)
    for n in (65, 100, 128, 200):
        B = rng.uniform(-1, 1, (A["n_cols"], n)).astype(dtype)
        for P in (0, 7):
            _check(A, B, P, f"wide{n}")
    # a leading dimension wider than n, and a row that spans many partitions
    c = np.stack([np.full(3000, 5, np.int64), np.arange(3000)], 1)
    pos, crd = to_csr(c, 9)
    A1 = {"n_rows": 9, "n_cols": 3000, "pos": pos, "crd": crd, "val": rng.uniform(-1, 1, 3000).astype(dtype)}
    Bfull = dev(rng.uniform(-1, 1, (3000, 160)).astype(dtype))
    Cfull = torch.full((9, 170), float("nan"), dtype=Bfull.dtype, device="cuda")
    nb.nacho_spmm(csr_operand(A1), Bfull[:, :150], Cfull[:, :150], P=40)
    torch.cuda.synchronize()
    ref, sabs = oracle.spmm(A1["pos"], A1["crd"], A1["val"], Bfull[:, :150].cpu().numpy())
    got = Cfull.cpu().numpy()
    assert tol_ok(got[:, :150], ref, sabs, TOL[dtype]).all()
    assert np.isnan(got[:, 150:]).all(), "columns beyond n were written"
