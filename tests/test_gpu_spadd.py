"""GPU parity: nacho_spadd_k vs the oracle's k-finger union merge.  Index arrays
(crd, pos, crd0, counts) must be bit-exact; values within 1e-5 (fp32) / 1e-12
(fp64) of the oracle's double sum, relative to max(|ref|, sum of |terms|)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_17198_amd import binding as nb
from paper_2604_17198_amd import workloads
from gpu_util import dev
from util import random_coords, to_csr, to_dcsr, to_vector, tol_ok

pytestmark = pytest.mark.gpu

TOL = {np.float32: 1e-5, np.float64: 1e-12}


def _finish(out):
    torch.cuda.synchronize()
    rows, nnz = (int(v) for v in out.counts.cpu().numpy()[:2])
    return rows, nnz, int(out.status.cpu().numpy()[0])


def _vals_ok(got, ref, sabs, dtype, tag):
    ok = tol_ok(got, ref, sabs, TOL[dtype])
    assert ok.all(), (tag, int((~ok).sum()))


def run_vec(vs, vals, extent, P, cap=None):
    dtype = vals[0].dtype.type
    ops = [nb.vector(dev(i), extent, dev(v)) for i, v in zip(vs, vals)]
    total = sum(len(i) for i in vs)
    out = nb.SparseOut("vector", 0, total if cap is None else cap, dev(vals[0]).dtype, "cuda")
    nb.nacho_spadd_k(ops, out, P=P)
    rows, nnz, status = _finish(out)
    return out, nnz, status


def check_vec(vs, vals, extent, P, tag):
    print(f"spadd vec {tag} k={len(vs)} sizes={[len(v) for v in vs]} P={P}", flush=True)
    out, nnz, status = run_vec(vs, vals, extent, P)
    ri, rv, ra = oracle.spadd_vec(vs, vals)
    assert status == 0 and nnz == ri.shape[0], (tag, status, nnz, ri.shape[0])
    assert np.array_equal(out.crd1.cpu().numpy()[:nnz], ri), tag
    assert out.pos1.cpu().numpy().tolist() == [0, nnz]
    _vals_ok(out.val.cpu().numpy()[:nnz], rv, ra, vals[0].dtype.type, tag)


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5, 8])
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_vectors_random(k, dtype):
    rng = np.random.default_rng(300 + k)
    for trial in range(5):
        extent = int(rng.choice([50, 5000, 10**6, 2**30]))
        vs, vals = [], []
        for t in range(k):
            n = int(rng.integers(0, min(extent, 20000) + 1))
            idx = np.unique(rng.integers(0, extent, n)).astype(np.int32)
            if trial == 1 and t > 0:
                idx = vs[0].copy()                       # all coordinates tied
            if trial == 2 and t == 1:
                idx = np.zeros(0, np.int32)              # an empty operand
            vs.append(idx)
            vals.append(rng.uniform(-1, 1, idx.shape[0]).astype(dtype))
        for P in (0, 1, 13, 500):
            check_vec(vs, vals, extent, P, f"random{trial}")


def test_vector_capacity_overflow_is_reported():
    rng = np.random.default_rng(5)
    vs = [np.unique(rng.integers(0, 10**6, 5000)).astype(np.int32) for _ in range(2)]
    vals = [rng.uniform(-1, 1, len(v)).astype(np.float32) for v in vs]
    ri, _, _ = oracle.spadd_vec(vs, vals)
    out, nnz, status = run_vec(vs, vals, 10**6, 0, cap=ri.shape[0] - 7)
    assert status == -4 and nnz == ri.shape[0]
    out, nnz, status = run_vec(vs, vals, 10**6, 0, cap=ri.shape[0])
    assert status == 0 and np.array_equal(out.crd1.cpu().numpy()[:nnz], ri)


def _mat_case(rng, shape, k, nmax, dtype):
    mats = []
    for t in range(k):
        n = int(rng.integers(0, min(shape[0] * shape[1], nmax) + 1))
        c = random_coords(rng, shape, n)
        mats.append((c, rng.uniform(-1, 1, c.shape[0]).astype(dtype)))
    return mats


def check_dcsr(mats, shape, P, tag):
    dtype = mats[0][1].dtype.type
    print(f"spadd dcsr {tag} k={len(mats)} shape={shape} sizes={[m[0].shape[0] for m in mats]} P={P}", flush=True)
    gops, omats = [], []
    for c, v in mats:
        p0, c0, p1, c1 = to_dcsr(c)
        gops.append(nb.dcsr(dev(p0), dev(c0), dev(p1), dev(c1), shape[0], shape[1], dev(v)))
        omats.append({"pos0": p0, "crd0": c0, "pos1": p1, "crd1": c1, "val": v})
    cap_r = sum(m["crd0"].shape[0] for m in omats)
    cap_n = sum(m["crd1"].shape[0] for m in omats)
    out = nb.SparseOut("dcsr", cap_r, cap_n, dev(mats[0][1]).dtype, "cuda")
    nb.nacho_spadd_k(gops, out, P=P)
    rows, nnz, status = _finish(out)
    ref = oracle.spadd_dcsr(omats)
    assert status == 0 and rows == ref["crd0"].shape[0] and nnz == ref["crd1"].shape[0], tag
    assert np.array_equal(out.pos0.cpu().numpy(), ref["pos0"]), tag
    assert np.array_equal(out.crd0.cpu().numpy()[:rows], ref["crd0"]), tag
    assert np.array_equal(out.pos1.cpu().numpy()[:rows + 1], ref["pos1"]), tag
    assert np.array_equal(out.crd1.cpu().numpy()[:nnz], ref["crd1"]), tag
    _vals_ok(out.val.cpu().numpy()[:nnz], ref["val"], ref["abs"], dtype, tag)


def check_csr(mats, shape, P, tag):
    dtype = mats[0][1].dtype.type
    print(f"spadd csr {tag} k={len(mats)} shape={shape} sizes={[m[0].shape[0] for m in mats]} P={P}", flush=True)
    gops, omats = [], []
    for c, v in mats:
        pos, crd = to_csr(c, shape[0])
        gops.append(nb.csr(dev(pos), dev(crd), shape[0], shape[1], dev(v)))
        omats.append({"pos": pos, "crd": crd, "val": v})
    cap_n = sum(m["crd"].shape[0] for m in omats)
    out = nb.SparseOut("csr", 0, cap_n, dev(mats[0][1]).dtype, "cuda", n_rows=shape[0])
    out.pos1.fill_(-7)
    nb.nacho_spadd_k(gops, out, P=P)
    rows, nnz, status = _finish(out)
    ref = oracle.spadd_csr(omats)
    assert status == 0 and rows == shape[0] and nnz == ref["crd"].shape[0], tag
    assert np.array_equal(out.pos1.cpu().numpy(), ref["pos"]), tag
    assert np.array_equal(out.crd1.cpu().numpy()[:nnz], ref["crd"]), tag
    _vals_ok(out.val.cpu().numpy()[:nnz], ref["val"], ref["abs"], dtype, tag)


@pytest.mark.parametrize("k", [1, 2, 3, 4])
@pytest.mark.parametrize("fmt", ["dcsr", "csr"])
def test_matrices_random(fmt, k):
    rng = np.random.default_rng(400 + k)
    check = check_dcsr if fmt == "dcsr" else check_csr
    for trial in range(5):
        shape = (int(rng.integers(1, 3000)), int(rng.integers(1, 3000)))
        mats = _mat_case(rng, shape, k, 12000, np.float32 if trial % 2 else np.float64)
        if trial == 1 and k > 1:
            mats[1] = (mats[0][0].copy(), mats[1][1][:0].copy())
            mats[1] = (mats[0][0].copy(), rng.uniform(-1, 1, mats[0][0].shape[0]).astype(mats[0][1].dtype))
        for P in (0, 1, 9, 700):
            check(mats, shape, P, f"{fmt}{trial}")


@pytest.mark.parametrize("k", [2, 3, 5, 8])
def test_dcsr_short_rows_many_operands(k):
    """Rows of one to three entries, shared by many operands, equal sizes (every run searches and
    is searched): where a row of the output starts is settled by the searches of the ranking."""
    rng = np.random.default_rng(70 + k)
    for shape, dens in (((6000, 3), 0.5), ((3000, 8), 0.3), ((20000, 2), 0.2)):
        mats = []
        for t in range(k):
            c = random_coords(rng, shape, int(dens * shape[0] * shape[1]))
            mats.append((c, rng.uniform(-1, 1, c.shape[0]).astype(np.float32)))
        for P in (0, 3, 50):
            check_dcsr(mats, shape, P, f"short rows {shape}")


def test_degenerate_matrices():
    rng = np.random.default_rng(9)
    z = np.zeros((0, 2), np.int64)
    zv = np.zeros(0, np.float32)
    one_row = np.stack([np.full(3000, 5, np.int64), np.arange(3000)], 1)
    one_col = np.stack([np.arange(2500), np.full(2500, 3, np.int64)], 1)
    v = lambda c: rng.uniform(-1, 1, c.shape[0]).astype(np.float32)
    for check in (check_dcsr, check_csr):
        check([(z, zv), (z, zv)], (40, 50), 0, "all-empty")
        check([(z, zv), (one_row, v(one_row))], (40, 3000), 0, "empty+row")
        check([(one_row, v(one_row)), (one_row, v(one_row)), (one_col[:40], v(one_col[:40]))], (40, 3000), 0, "rows")
        check([(one_col, v(one_col)), (one_col, v(one_col))], (2500, 9), 7, "cols")


def test_config3_scaled():
    cfg = workloads.config(3, scale=0.03)
    vs = [o["i"] for o in cfg["ops"]]
    vals = [o["v"] for o in cfg["ops"]]
    check_vec(vs, vals, cfg["extent"], 0, "config3@0.03")


def test_config4_scaled():
    cfg = workloads.config(4, scale=0.02)
    mats = []
    for m in cfg["ops"]:
        rows = np.repeat(m["crd0"].astype(np.int64), np.diff(m["pos1"]))
        mats.append((np.stack([rows, m["crd1"].astype(np.int64)], 1), m["val"]))
    check_dcsr(mats, (cfg["n_rows"], cfg["n_cols"]), 0, "config4@0.02")


def test_config3_full_size():
    cfg = workloads.config(3)
    vs = [o["i"] for o in cfg["ops"]]
    vals = [o["v"] for o in cfg["ops"]]
    check_vec(vs, vals, cfg["extent"], 0, "config3 full")


def test_config4_full_size():
    cfg = workloads.config(4)
    A, B = cfg["ops"]
    gops = [nb.dcsr(dev(m["pos0"]), dev(m["crd0"]), dev(m["pos1"]), dev(m["crd1"]),
                    m["n_rows"], m["n_cols"], dev(m["val"])) for m in (A, B)]
    cap_r = A["crd0"].shape[0] + B["crd0"].shape[0]
    cap_n = A["crd1"].shape[0] + B["crd1"].shape[0]
    print(f"spadd dcsr config4 full nnz={cap_n}", flush=True)
    out = nb.SparseOut("dcsr", cap_r, cap_n, torch.float32, "cuda")
    nb.nacho_spadd_k(gops, out)
    rows, nnz, status = _finish(out)
    ref = oracle.spadd_dcsr([A, B])
    assert status == 0 and rows == ref["crd0"].shape[0] and nnz == ref["crd1"].shape[0]
    assert np.array_equal(out.crd0.cpu().numpy()[:rows], ref["crd0"])
    assert np.array_equal(out.pos1.cpu().numpy()[:rows + 1], ref["pos1"])
    assert np.array_equal(out.crd1.cpu().numpy()[:nnz], ref["crd1"])
    _vals_ok(out.val.cpu().numpy()[:nnz], ref["val"], ref["abs"], np.float32, "config4 full")


@pytest.mark.parametrize("k", [2, 3])
def test_csr_add_powerlaw_full_size(k):
    """Fused k-way CSR addition on power-law matrices of the paper's skew-experiment shape
    (100000 x 100000, 5M non-zeros each), against the oracle's k-finger union."""
    cfg = workloads.csr_add_config(k)
    mats = cfg["ops"]
    print(f"spadd csr powerlaw k={k} nnz={[int(m['pos'][-1]) for m in mats]}", flush=True)
    gops = [nb.csr(dev(m["pos"]), dev(m["crd"]), m["n_rows"], m["n_cols"], dev(m["val"])) for m in mats]
    total = sum(int(m["pos"][-1]) for m in mats)
    out = nb.SparseOut("csr", 0, total, torch.float32, "cuda", n_rows=cfg["n_rows"])
    nb.nacho_spadd_k(gops, out)
    rows, nnz, status = _finish(out)
    ref = oracle.spadd_csr([{"pos": m["pos"], "crd": m["crd"], "val": m["val"]} for m in mats])
    assert status == 0 and rows == cfg["n_rows"] and nnz == ref["crd"].shape[0]
    assert np.array_equal(out.pos1.cpu().numpy(), ref["pos"])
    assert np.array_equal(out.crd1.cpu().numpy()[:nnz], ref["crd"])
    _vals_ok(out.val.cpu().numpy()[:nnz], ref["val"], ref["abs"], np.float32, f"csr add k={k}")
