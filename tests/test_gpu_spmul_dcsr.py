"""GPU parity: nacho_spmul_k on DCSR operands (outer intersection, recursive
partitioning of Section 3.3) vs the oracle.  Index arrays and the stored
partitions of the remapped nest bit-exact; values within 1e-5 (fp32) / 1e-12
(fp64) relative to |ref| (a product has no cancellation)."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2604_17198_amd import binding as nb
from paper_2604_17198_amd import workloads
from gpu_util import dev
from util import random_coords, to_dcsr, tol_ok

pytestmark = pytest.mark.gpu

TOL = {np.float32: 1e-5, np.float64: 1e-12}


def _mat(coords, vals):
    coords = np.asarray(coords, dtype=np.int64).reshape(-1, 2)
    p0, c0, p1, c1 = to_dcsr(coords)
    return {"pos0": p0, "crd0": c0, "pos1": p1, "crd1": c1, "val": vals}


def run(mats, shape, P, tag, cap_rows=None, cap_nnz=None, check_parts=True):
    k = len(mats)
    print(f"spmul dcsr {tag} k={k} shape={shape} rows={[len(m['crd0']) for m in mats]} "
          f"nnz={[len(m['crd1']) for m in mats]} P={P}", flush=True)
    dtype = mats[0]["val"].dtype.type
    ops = [nb.dcsr(dev(m["pos0"]), dev(m["crd0"]), dev(m["pos1"]), dev(m["crd1"]), shape[0], shape[1],
                   dev(m["val"])) for m in mats]
    cr = min(len(m["crd0"]) for m in mats) if cap_rows is None else cap_rows
    cn = min(len(m["crd1"]) for m in mats) if cap_nnz is None else cap_nnz
    tdt = torch.float32 if dtype == np.float32 else torch.float64
    out = nb.SparseOut("dcsr", cr, cn, tdt, "cuda")
    out.pos1.fill_(-7)
    dt = nb.dtype_code(tdt)
    ws = torch.empty(nb.workspace_bytes(nb.OP_SPMUL, ops, dt, 0, P), dtype=torch.uint8, device="cuda")
    nb.nacho_spmul_k(ops, out, P=P, ws=ws)
    torch.cuda.synchronize()
    rows, nnz = (int(v) for v in out.counts.cpu().numpy()[:2])
    status = int(out.status.cpu().numpy()[0])
    ref = oracle.spmul_dcsr(mats)
    parts = None
    if check_parts and k > 1:
        parts = nb.workspace_parts(nb.OP_SPMUL, ops, dt, ws, 0, P)
        parts = {kk: (v.cpu().numpy() if torch.is_tensor(v) else v) for kk, v in parts.items()}
    return out, rows, nnz, status, ref, parts


def check(mats, shape, P, tag):
    out, rows, nnz, status, ref, parts = run(mats, shape, P, tag)
    k = len(mats)
    dtype = mats[0]["val"].dtype.type
    assert status == 0, (tag, status)
    assert rows == ref["crd0"].shape[0] and nnz == ref["crd1"].shape[0], (tag, rows, nnz)
    assert out.pos0.cpu().numpy().tolist() == [0, rows], tag
    assert np.array_equal(out.crd0.cpu().numpy()[:rows], ref["crd0"]), tag
    assert np.array_equal(out.pos1.cpu().numpy()[:rows + 1], ref["pos1"]), tag
    assert np.array_equal(out.crd1.cpu().numpy()[:nnz], ref["crd1"]), tag
    ok = tol_ok(out.val.cpu().numpy()[:nnz], ref["val"], ref["abs"], TOL[dtype])
    assert ok.all(), (tag, int((~ok).sum()))
    if parts is None:
        return None
    # the stored partitions are those of Algorithm 2 on the remapped nest
    Pe = parts["P"]
    if Pe == 0:                      # nothing to coiterate: no row in common or no entry in such rows
        r = oracle.recursive_partition_dcsr(mats, shape[1], 1)
        assert int(r["cost"][-1]) == 0, tag
        return parts
    r = oracle.recursive_partition_dcsr(mats, shape[1], Pe)
    M = r["rows"].shape[0]
    assert np.array_equal(parts["cost"], r["cost"]), tag
    assert np.array_equal(parts["coord"], r["coord"]), tag
    assert np.array_equal(parts["posn"][:, :, 1], r["before"]), tag
    assert np.array_equal(parts["posn"][:, :, 0], np.repeat(r["coord"][:, :1], k, axis=1)), tag
    assert int(parts["coord"][-1, 0]) == M
    return parts


def test_fig3b_example():
    """Figure 3(b): the chunks of the DCSR multiplication, four threads."""
    with open(os.path.join(os.path.dirname(__file__), "golden", "fig3b_dcsr_mul_partition.json")) as f:
        g = json.load(f)
    for dtype in (np.float32, np.float64):
        A = _mat(g["A"], np.arange(1, 13, dtype=dtype))
        B = _mat(g["B"], np.arange(2, 14, dtype=dtype))
        parts = check([A, B], (g["n_rows"], g["n_cols"]), g["P"], "fig3b")
        assert parts["P"] == g["P"]
        assert np.diff(parts["cost"]).tolist() == [4, 4, 4, 4]
        for t, key in enumerate(("A_membership", "B_membership")):
            memb = np.array(g[key])
            counts = np.bincount(memb[memb >= 0], minlength=g["P"])
            assert parts["posn"][:, t, 1].tolist() == [0] + np.cumsum(counts).tolist()


@pytest.mark.parametrize("k", [1, 2, 3, 4, 8])
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_random_small(k, dtype):
    rng = np.random.default_rng(900 + k)
    for trial in range(6):
        shape = [(30, 40), (200, 64), (64, 3000), (500, 500), (40, 40), (1000, 20)][trial]
        mats = []
        for t in range(k):
            dens = [0.5, 0.3, 0.1, 0.05, 0.9, 0.6][trial]
            c = random_coords(rng, shape, int(dens * shape[0] * shape[1]))
            if trial % 2 == 1:                   # drop rows, differently per operand: rows are skipped
                keep = rng.random(shape[0]) > 0.3
                c = c[keep[c[:, 0]]]
            v = (rng.uniform(0.5, 1.5, c.shape[0]) * rng.choice([-1, 1], c.shape[0])).astype(dtype)
            mats.append(_mat(c, v))
        for P in (0, 1, 7, 300):
            check(mats, shape, P, f"random{trial}")


def test_degenerate_inputs():
    rng = np.random.default_rng(4)
    shape = (50, 60)
    f32 = np.float32
    full = random_coords(rng, shape, 900)
    A = _mat(full, np.ones(full.shape[0], f32))
    empty = _mat(np.zeros((0, 2), np.int64), np.zeros(0, f32))
    check([A, empty], shape, 0, "one empty operand")
    check([empty, A], shape, 3, "first operand empty")
    check([empty, empty], shape, 0, "both empty")
    # no row in common
    ca = full[full[:, 0] % 2 == 0]
    cb = full[full[:, 0] % 2 == 1]
    check([_mat(ca, np.ones(len(ca), f32)), _mat(cb, np.ones(len(cb), f32))], shape, 0, "disjoint rows")
    # rows in common, no column in common: every result row is empty and none is stored
    ca = full[full[:, 1] % 2 == 0]
    cb = full[full[:, 1] % 2 == 1]
    check([_mat(ca, np.ones(len(ca), f32)), _mat(cb, np.ones(len(cb), f32))], shape, 5, "disjoint columns")
    # identical operands: every coordinate ties
    check([A, A, A], shape, 4, "identical")
    # a single common row that is long: many partitions inside one row
    c = np.stack([np.full(20000, 7), np.arange(20000)], axis=1)
    c2 = np.concatenate([np.stack([np.full(100, 3), np.arange(100)], axis=1), c[::2]])
    check([_mat(c, np.ones(len(c), f32)), _mat(c2, np.full(len(c2), 2, f32))], (10, 20000), 0, "one long row")


@pytest.mark.parametrize("k", [2, 3])
def test_medium_many_tiles(k):
    """Several scan tiles of rows and many partitions; half of the stored rows are shared."""
    rng = np.random.default_rng(31 + k)
    n = 60000
    shape = (n, 4000)
    shared = rng.choice(n, 9000, replace=False)
    mats = []
    for t in range(k):
        own = rng.choice(n, 9000, replace=False)
        rows = np.unique(np.concatenate([shared, own]))
        lens = rng.integers(1, 60, rows.shape[0])
        lens[rng.integers(0, rows.shape[0], 5)] = 3000          # a few long rows
        rr = np.repeat(rows, lens)
        cc = np.concatenate([np.sort(rng.choice(shape[1], l, replace=False)) for l in lens])
        v = rng.uniform(0.5, 1.5, rr.shape[0]).astype(np.float32)
        mats.append(_mat(np.stack([rr, cc], axis=1), v))
    for P in (0, 1000):
        check(mats, shape, P, "medium")


def test_capacity_overflow_is_reported():
    rng = np.random.default_rng(8)
    shape = (300, 200)
    cs = [random_coords(rng, shape, 20000) for _ in range(2)]
    mats = [_mat(c, np.ones(len(c), np.float32)) for c in cs]
    ref = oracle.spmul_dcsr(mats)
    nr, nz = ref["crd0"].shape[0], ref["crd1"].shape[0]
    out, rows, nnz, status, _, _ = run(mats, shape, 0, "cap nnz", cap_nnz=nz - 5, check_parts=False)
    assert status == -4 and (rows, nnz) == (nr, nz)
    assert np.array_equal(out.crd1.cpu().numpy()[:nz - 5], ref["crd1"][:nz - 5])
    out, rows, nnz, status, _, _ = run(mats, shape, 0, "cap rows", cap_rows=nr - 3, check_parts=False)
    assert status == -4 and (rows, nnz) == (nr, nz)
    assert np.array_equal(out.crd0.cpu().numpy()[:nr - 3], ref["crd0"][:nr - 3])


def test_workspace_too_small_and_reuse():
    rng = np.random.default_rng(12)
    shape = (100, 100)
    cs = [random_coords(rng, shape, 3000) for _ in range(2)]
    mats = [_mat(c, np.ones(len(c), np.float64)) for c in cs]
    ops = [nb.dcsr(dev(m["pos0"]), dev(m["crd0"]), dev(m["pos1"]), dev(m["crd1"]), *shape, dev(m["val"]))
           for m in mats]
    out = nb.SparseOut("dcsr", 100, 3000, torch.float64, "cuda")
    need = nb.workspace_bytes(nb.OP_SPMUL, ops, nb.dtype_code(torch.float64), 0, 0)
    small = torch.empty(need - 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(nb.NachoError) as e:
        nb.nacho_spmul_k(ops, out, ws=small)
    assert e.value.status == -3
    # the same workspace serves calls in a row (a smaller product after a larger one)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    ref = oracle.spmul_dcsr(mats)
    for rep in range(2):
        nb.nacho_spmul_k(ops, out, ws=ws)
        torch.cuda.synchronize()
        assert out.counts.cpu().numpy()[:2].tolist() == [ref["crd0"].shape[0], ref["crd1"].shape[0]]
        assert np.array_equal(out.crd1.cpu().numpy()[:ref["crd1"].shape[0]], ref["crd1"])


def test_the_call_only_enqueues():
    """The sizes of the remapped space stay on the device: the call comes back while the stream is
    still busy with work queued before it, and the result is right once the stream has drained."""
    cfg = workloads.config(4, scale=0.05)
    mats = [{kk: m[kk] for kk in ("pos0", "crd0", "pos1", "crd1", "val")} for m in cfg["ops"]]
    shape = (cfg["n_rows"], cfg["n_cols"])
    ops = [nb.dcsr(dev(m["pos0"]), dev(m["crd0"]), dev(m["pos1"]), dev(m["crd1"]), shape[0], shape[1],
                   dev(m["val"])) for m in mats]
    out = nb.SparseOut("dcsr", min(len(m["crd0"]) for m in mats), min(len(m["crd1"]) for m in mats),
                       torch.float32, "cuda")
    ws = torch.empty(nb.workspace_bytes(nb.OP_SPMUL, ops, nb.F32), dtype=torch.uint8, device="cuda")
    a = torch.randn(8192, 8192, device="cuda")
    torch.cuda.synchronize()
    print("spmul dcsr behind a busy stream", flush=True)
    for _ in range(12):
        a = (a @ a) * 1e-4                      # tens of milliseconds of work ahead of the call
    nb.nacho_spmul_k(ops, out, ws=ws)
    done = torch.cuda.Event()
    done.record()
    assert not done.query(), "the call waited for the stream"
    torch.cuda.synchronize()
    ref = oracle.spmul_dcsr(mats)
    assert out.counts.cpu().numpy()[:2].tolist() == [ref["crd0"].shape[0], ref["crd1"].shape[0]]
    assert int(out.status.cpu().numpy()[0]) == 0
    assert np.array_equal(out.crd1.cpu().numpy()[:ref["crd1"].shape[0]], ref["crd1"])
    assert np.array_equal(out.crd0.cpu().numpy()[:ref["crd0"].shape[0]], ref["crd0"])


def test_config4_operands_full_size():
    """The two DCSR matrices of configuration 4 multiplied: half of each operand's rows are skipped."""
    cfg = workloads.config(4)
    mats = [{kk: m[kk] for kk in ("pos0", "crd0", "pos1", "crd1", "val")} for m in cfg["ops"]]
    parts = check(mats, (cfg["n_rows"], cfg["n_cols"]), 0, "config4 full")
    w = np.diff(parts["cost"])
    assert w.max() <= 4096 and w.max() - w.min() <= 4
