"""GPU parity: nacho_spmv vs the oracle (plain y_i = sum_j A_ij x_j accumulated
in long double).  Tolerance: |y - y_ref| <= tol * max(|y_ref|, sum_j |A_ij x_j|)
with tol = 1e-12 (fp64) and 1e-5 (fp32); empty rows must be exactly 0."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_17198_amd import binding as nb
from paper_2604_17198_amd import workloads
from gpu_util import csr_operand, dev
from util import random_coords, to_csr, tol_ok

pytestmark = pytest.mark.gpu

TOL = {np.float64: 1e-12, np.float32: 1e-5}


def _run(A, x, P):
    y = torch.full((A["n_rows"],), float("nan"), dtype=dev(x).dtype, device="cuda")
    nb.nacho_spmv(csr_operand(A), dev(x), y, P=P)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def _check(A, x, P, tag):
    dtype = A["val"].dtype.type
    print(f"spmv {tag} rows={A['n_rows']} nnz={int(A['pos'][-1])} P={P} dtype={dtype.__name__}", flush=True)
    y = _run(A, x, P)
    ref, s = oracle.spmv(A["pos"], A["crd"], A["val"], x)
    assert not np.any(np.isnan(y)), f"{tag}: some y[i] never written"
    ok = tol_ok(y, ref, s, TOL[dtype])
    assert ok.all(), (tag, int((~ok).sum()), np.abs(y - ref)[~ok][:5], ref[~ok][:5])
    assert np.all(y[np.diff(A["pos"]) == 0] == 0.0)
    return y


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_random_small(dtype):
    rng = np.random.default_rng(1)
    for trial in range(10):
        n_rows, n_cols = int(rng.integers(1, 3000)), int(rng.integers(1, 3000))
        nnz = int(rng.integers(0, min(n_rows * n_cols, 20000) + 1))
        c = random_coords(rng, (n_rows, n_cols), nnz)
        pos, crd = to_csr(c, n_rows)
        A = {"n_rows": n_rows, "n_cols": n_cols, "pos": pos, "crd": crd,
             "val": rng.uniform(-1, 1, nnz).astype(dtype)}
        x = rng.uniform(-1, 1, n_cols).astype(dtype)
        for P in (0, 1, 7, nnz + 5):
            _check(A, x, P, f"random{trial}")


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_degenerate_shapes(dtype):
    rng = np.random.default_rng(2)
    # all-empty matrix, single dense row, single column, one heavy row among empties
    cases = {
        "empty": np.zeros((0, 2), np.int64),
        "one_row": np.stack([np.zeros(5000, np.int64), np.arange(5000)], 1),
        "one_col": np.stack([np.arange(3000), np.zeros(3000, np.int64)], 1),
        "heavy_mid": np.stack([np.full(9000, 1234, np.int64), np.arange(9000)], 1),
    }
    shapes = {"empty": (777, 5), "one_row": (1, 5000), "one_col": (3000, 1), "heavy_mid": (5000, 9000)}
    for name, c in cases.items():
        n_rows, n_cols = shapes[name]
        pos, crd = to_csr(c, n_rows)
        A = {"n_rows": n_rows, "n_cols": n_cols, "pos": pos, "crd": crd,
             "val": rng.uniform(-1, 1, c.shape[0]).astype(dtype)}
        x = rng.uniform(-1, 1, n_cols).astype(dtype)
        for P in (0, 3, 40):
            _check(A, x, P, name)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_long_runs_of_empty_rows(dtype):
    """A few stored rows among hundreds of thousands of empty ones (at the start, between stored
    rows, at the end): the empty rows are exactly 0 and cost the executing wavefronts nothing."""
    rng = np.random.default_rng(5)
    n_rows, n_cols = 700_000, 4000
    lens = {150_000: 3000, 150_001: 1, 150_700: 40, 420_000: 2500, 420_513: 7, 699_998: 600}
    rows = np.repeat(list(lens), list(lens.values()))
    cols = np.concatenate([np.sort(rng.choice(n_cols, l, replace=False)) for l in lens.values()])
    pos, crd = to_csr(np.stack([rows, cols], 1), n_rows)
    A = {"n_rows": n_rows, "n_cols": n_cols, "pos": pos, "crd": crd,
         "val": rng.uniform(-1, 1, crd.shape[0]).astype(dtype)}
    x = rng.uniform(-1, 1, n_cols).astype(dtype)
    for P in (0, 1, 5, 64):
        _check(A, x, P, "empty runs")


def test_config1_all_partition_counts():
    cfg = workloads.config(1)
    for P in (0, 1, 20, 333, 50_000):          # 50_000 > nnz: repeated boundaries
        _check(cfg["A"], cfg["x"], P, "config1")


def test_bitwise_repeatable():
    cfg = workloads.config(2, scale=0.02)
    y1 = _run(cfg["A"], cfg["x"], 0)
    y2 = _run(cfg["A"], cfg["x"], 0)
    assert np.array_equal(y1.view(np.int64), y2.view(np.int64))


def test_config2_scaled_and_fp32():
    cfg = workloads.config(2, scale=0.05)
    _check(cfg["A"], cfg["x"], 0, "config2@0.05")
    A32 = dict(cfg["A"], val=cfg["A"]["val"].astype(np.float32))
    _check(A32, cfg["x"].astype(np.float32), 0, "config2@0.05 fp32")


def test_config2_full_size():
    cfg = workloads.config(2)
    _check(cfg["A"], cfg["x"], 0, "config2 full")


def test_errors_from_the_host():
    cfg = workloads.config(1)
    A, x = csr_operand(cfg["A"]), dev(cfg["x"])
    y = torch.empty(cfg["A"]["n_rows"], dtype=torch.float64, device="cuda")
    tiny = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(nb.NachoError) as e:
        nb.nacho_spmv(A, x, y, ws=tiny)
    assert e.value.status == -3
    with pytest.raises(nb.NachoError) as e:                  # misaligned val
        bad = nb.csr(A.keep[0], A.keep[1], 4096, 4096, A.val[1:])
        nb.nacho_spmv(bad, x, y)
    assert e.value.status == -1


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_fused_search_in_execute_variant(dtype):
    """nacho_spmv_fused has no partition pass: every wavefront searches its own boundaries.  Same
    partitions and arithmetic as nacho_spmv with P = 0, so the results agree bit for bit; and with
    the oracle within the tolerance."""
    rng = np.random.default_rng(8)
    mats = []
    for trial in range(6):
        n_rows, n_cols = int(rng.integers(1, 4000)), int(rng.integers(1, 4000))
        nnz = int(rng.integers(0, min(n_rows * n_cols, 40000) + 1))
        c = random_coords(rng, (n_rows, n_cols), nnz)
        if trial % 2:
            c = c[c[:, 0] % 7 != 3]                   # runs of empty rows
        pos, crd = to_csr(c, n_rows)
        mats.append(({"n_rows": n_rows, "n_cols": n_cols, "pos": pos, "crd": crd,
                      "val": rng.uniform(-1, 1, c.shape[0]).astype(dtype)},
                     rng.uniform(-1, 1, n_cols).astype(dtype), f"random{trial}"))
    # all-empty matrix, one row spanning many partitions among empty rows, the skewed configuration
    pos, crd = to_csr(np.zeros((0, 2), np.int64), 300)
    mats.append(({"n_rows": 300, "n_cols": 9, "pos": pos, "crd": crd, "val": np.zeros(0, dtype)},
                 rng.uniform(-1, 1, 9).astype(dtype), "empty"))
    c = np.stack([np.full(30000, 4321, np.int64), np.arange(30000)], 1)
    pos, crd = to_csr(c, 9000)
    mats.append(({"n_rows": 9000, "n_cols": 30000, "pos": pos, "crd": crd,
                  "val": rng.uniform(-1, 1, 30000).astype(dtype)}, rng.uniform(-1, 1, 30000).astype(dtype), "heavy"))
    cfg = workloads.config(2, scale=0.05)
    mats.append((dict(cfg["A"], val=cfg["A"]["val"].astype(dtype)), cfg["x"].astype(dtype), "config2@0.05"))
    for A, x, tag in mats:
        print(f"spmv fused {tag} rows={A['n_rows']} nnz={int(A['pos'][-1])} {np.dtype(dtype).name}", flush=True)
        op, xd = csr_operand(A), dev(x)
        y = torch.full((A["n_rows"],), float("nan"), dtype=xd.dtype, device="cuda")
        nb.nacho_spmv_fused(op, xd, y)
        torch.cuda.synchronize()
        got = y.cpu().numpy()
        ref, s = oracle.spmv(A["pos"], A["crd"], A["val"], x)
        assert not np.any(np.isnan(got)), tag
        assert tol_ok(got, ref, s, TOL[dtype]).all(), tag
        assert np.all(got[np.diff(A["pos"]) == 0] == 0.0)
        plain = _run(A, x, 0)
        assert np.array_equal(got.view(np.uint8), plain.view(np.uint8)), tag
