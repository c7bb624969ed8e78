"""GPU parity: nacho_spmul_k (k-way intersection with products) vs the oracle's
k-finger intersection.  Index arrays bit-exact; values within 1e-5 (fp32) /
1e-12 (fp64) relative to |ref| (a product of k factors has no cancellation)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_17198_amd import binding as nb
from paper_2604_17198_amd import workloads
from gpu_util import dev
from util import random_coords, to_csr, tol_ok

pytestmark = pytest.mark.gpu

TOL = {np.float32: 1e-5, np.float64: 1e-12}


def _finish(out):
    torch.cuda.synchronize()
    rows, nnz = (int(v) for v in out.counts.cpu().numpy()[:2])
    return rows, nnz, int(out.status.cpu().numpy()[0])


def check_vec(vs, vals, extent, P, tag, cap=None):
    print(f"spmul vec {tag} k={len(vs)} sizes={[len(v) for v in vs]} P={P}", flush=True)
    dtype = vals[0].dtype.type
    ops = [nb.vector(dev(i), extent, dev(v)) for i, v in zip(vs, vals)]
    out = nb.SparseOut("vector", 0, min(len(i) for i in vs) if cap is None else cap, dev(vals[0]).dtype, "cuda")
    nb.nacho_spmul_k(ops, out, P=P)
    rows, nnz, status = _finish(out)
    ri, rv, ra = oracle.spmul_vec(vs, vals)
    assert status == 0 and nnz == ri.shape[0], (tag, status, nnz, ri.shape[0])
    assert np.array_equal(out.crd1.cpu().numpy()[:nnz], ri), tag
    assert out.pos1.cpu().numpy().tolist() == [0, nnz]
    ok = tol_ok(out.val.cpu().numpy()[:nnz], rv, ra, TOL[dtype])
    assert ok.all(), (tag, int((~ok).sum()))


def check_csr(mats, shape, P, tag):
    print(f"spmul csr {tag} k={len(mats)} shape={shape} nnz={[len(m['crd']) for m in mats]} P={P}", flush=True)
    dtype = mats[0]["val"].dtype.type
    ops = [nb.csr(dev(m["pos"]), dev(m["crd"]), shape[0], shape[1], dev(m["val"])) for m in mats]
    out = nb.SparseOut("csr", 0, min(len(m["crd"]) for m in mats), dev(mats[0]["val"]).dtype, "cuda", n_rows=shape[0])
    out.pos1.fill_(-7)
    nb.nacho_spmul_k(ops, out, P=P)
    rows, nnz, status = _finish(out)
    ref = oracle.spmul_csr(mats)
    assert status == 0 and rows == shape[0] and nnz == ref["crd"].shape[0], (tag, status, nnz)
    assert np.array_equal(out.pos1.cpu().numpy(), ref["pos"]), tag
    assert np.array_equal(out.crd1.cpu().numpy()[:nnz], ref["crd"]), tag
    ok = tol_ok(out.val.cpu().numpy()[:nnz], ref["val"], ref["abs"], TOL[dtype])
    assert ok.all(), (tag, int((~ok).sum()))


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5, 8])
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_vectors_random(k, dtype):
    rng = np.random.default_rng(700 + k)
    for trial in range(5):
        extent = int(rng.choice([50, 5000, 40000]))
        vs, vals = [], []
        for t in range(k):
            n = int(rng.integers(extent // 3, extent + 1))       # dense enough for k-way matches
            idx = np.unique(rng.integers(0, extent, n)).astype(np.int32)
            if trial == 1 and t > 0:
                idx = vs[0].copy()                               # all coordinates tied
            if trial == 2 and t == k - 1 and k > 1:
                idx = np.zeros(0, np.int32)                      # an empty operand: empty result
            vs.append(idx)
            vals.append(rng.uniform(0.5, 1.5, idx.shape[0]).astype(dtype) * rng.choice([-1, 1], idx.shape[0]))
        vals = [v.astype(dtype) for v in vals]
        for P in (0, 1, 13, 500):
            check_vec(vs, vals, extent, P, f"random{trial}")


@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_csr_random(k):
    rng = np.random.default_rng(800 + k)
    for trial in range(5):
        shape = (int(rng.integers(1, 400)), int(rng.integers(1, 300)))
        dtype = np.float32 if trial % 2 else np.float64
        mats = []
        for t in range(k):
            nmax = shape[0] * shape[1]
            c = random_coords(rng, shape, int(rng.integers(nmax // 3, nmax * 9 // 10 + 1)))
            if trial == 1 and t > 0:
                c = random_coords(rng, shape, 0) if t == 1 else c
            pos, crd = to_csr(c, shape[0])
            mats.append({"pos": pos, "crd": crd, "val": rng.uniform(0.5, 1.5, crd.shape[0]).astype(dtype)})
        for P in (0, 1, 7, 300):
            check_csr(mats, shape, P, f"random{trial}")


def test_capacity_overflow_is_reported():
    rng = np.random.default_rng(9)
    vs = [np.unique(rng.integers(0, 20000, 15000)).astype(np.int32) for _ in range(2)]
    vals = [rng.uniform(0.5, 1.5, len(v)).astype(np.float32) for v in vs]
    ri, _, _ = oracle.spmul_vec(vs, vals)
    ops = [nb.vector(dev(i), 20000, dev(v)) for i, v in zip(vs, vals)]
    out = nb.SparseOut("vector", 0, ri.shape[0] - 5, torch.float32, "cuda")
    nb.nacho_spmul_k(ops, out)
    rows, nnz, status = _finish(out)
    assert status == -4 and nnz == ri.shape[0]
    assert np.array_equal(out.crd1.cpu().numpy()[:ri.shape[0] - 5], ri[:-5])


def test_config3_vectors_full_size():
    """The three vectors of configuration 3 multiplied: coordinates stored by all of a, b and c."""
    cfg = workloads.config(3)
    vs = [o["i"] for o in cfg["ops"]]
    vals = [o["v"] for o in cfg["ops"]]
    check_vec(vs, vals, cfg["extent"], 0, "config3 full")


def test_csr_hadamard_powerlaw_full_size():
    cfg = workloads.csr_add_config(2)
    mats = [{"pos": m["pos"], "crd": m["crd"], "val": m["val"]} for m in cfg["ops"]]
    check_csr(mats, (cfg["n_rows"], cfg["n_cols"]), 0, "powerlaw 100k")
