"""GPU parity: nacho_partition vs the oracle's Algorithm 1, bit-exact on every
boundary coordinate, position and cost."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_17198_amd import binding as nb
from paper_2604_17198_amd import workloads
from gpu_util import csr_operand, dcsr_operand, dev, parts_to_numpy, vector_operand
from util import random_coords, to_csf3, to_csr, to_dcsr, to_vector

pytestmark = pytest.mark.gpu


def _compare(got, ref, tag):
    assert np.array_equal(got["cost"], ref["cost"]), tag
    assert np.array_equal(got["posn"].astype(np.int64), ref["posn"]), tag
    assert np.array_equal(got["coord"].astype(np.int64), ref["coord"][:, :got["coord"].shape[1]]), tag


def _vec_ops(vs, extent):
    g = [nb.vector(dev(v), extent) for v in vs]
    o = [oracle.vector(v, extent) for v in vs]
    return g, o


@pytest.mark.parametrize("k", [1, 2, 3, 5, 8])
def test_vectors_random_small(k):
    rng = np.random.default_rng(100 + k)
    for trial in range(6):
        extent = int(rng.choice([1, 7, 300, 100_000, 2**31 - 1]))
        vs = []
        for t in range(k):
            n = int(rng.integers(0, min(extent, 3000) + 1))
            v = to_vector(random_coords(rng, (extent,), n)) if extent < 10**6 else \
                np.unique(rng.integers(0, extent, n)).astype(np.int32)
            if trial == 1 and t > 0:
                v = vs[0].copy()                       # every coordinate tied across operands
            vs.append(v)
        g, o = _vec_ops(vs, extent)
        total = sum(len(v) for v in vs)
        for P in (1, 2, 5, 64, 257, total + 3):
            print(f"partition vec k={k} trial={trial} extent={extent} total={total} P={P}", flush=True)
            got = parts_to_numpy(nb.nacho_partition(g, P))
            _compare(got, oracle.partition(o, P), (k, trial, P))


def test_vectors_explicit_queries_and_cost_scale():
    rng = np.random.default_rng(7)
    vs = [to_vector(random_coords(rng, (5000,), n)) for n in (900, 2000, 10)]
    g, o = _vec_ops(vs, 5000)
    total = 2910
    q = np.sort(rng.integers(0, total + 50, 41)).astype(np.int64)
    got = parts_to_numpy(nb.nacho_partition(g, 40, queries=dev(q)))
    _compare(got, oracle.partition(o, 40, queries=q), "explicit")
    # scaled cost: boundaries of floor(Q / scale), costs in scaled units
    scale = 64
    qs = (np.arange(41, dtype=np.int64) * (total * scale // 40) // scale) * scale
    got = parts_to_numpy(nb.nacho_partition(g, 40, queries=dev(qs), cost_scale=scale))
    ref = oracle.partition(o, 40, queries=qs // scale)
    assert np.array_equal(got["posn"].astype(np.int64), ref["posn"])
    assert np.array_equal(got["coord"].astype(np.int64), ref["coord"])
    assert np.array_equal(got["cost"][:-1], ref["cost"][:-1] * scale)


@pytest.mark.parametrize("fmt", ["csr", "dcsr"])
@pytest.mark.parametrize("k", [1, 2, 3])
def test_matrices_random_small(fmt, k):
    rng = np.random.default_rng(200 + k)
    for trial in range(6):
        shape = (int(rng.integers(1, 400)), int(rng.integers(1, 400)))
        g, o, total = [], [], 0
        for t in range(k):
            n = int(rng.integers(0, min(shape[0] * shape[1], 6000) + 1))
            c = random_coords(rng, shape, n)
            total += c.shape[0]
            if fmt == "csr":
                pos, crd = to_csr(c, shape[0])
                g.append(nb.csr(dev(pos), dev(crd), *shape))
                o.append(oracle.csr(pos, crd, *shape))
            else:
                p0, c0, p1, c1 = to_dcsr(c)
                g.append(nb.dcsr(dev(p0), dev(c0), dev(p1), dev(c1), *shape))
                o.append(oracle.dcsr(p0, c0, p1, c1, *shape))
        for P in (1, 3, 17, 300, total + 2):
            print(f"partition {fmt} k={k} trial={trial} shape={shape} total={total} P={P}", flush=True)
            got = parts_to_numpy(nb.nacho_partition(g, P))
            _compare(got, oracle.partition(o, P), (fmt, k, trial, P))


def test_config1_and_scaled_configs():
    c1 = workloads.config(1)
    A = c1["A"]
    for P in (20, 39, 4096):
        print(f"partition config1 P={P}", flush=True)
        got = parts_to_numpy(nb.nacho_partition([csr_operand(A)], P))
        _compare(got, oracle.partition([oracle.csr(A["pos"], A["crd"], A["n_rows"], A["n_cols"])], P), P)
    c3 = workloads.config(3, scale=0.02)
    print("partition config3 scaled", flush=True)
    got = parts_to_numpy(nb.nacho_partition([vector_operand(v) for v in c3["ops"]], 999))
    _compare(got, oracle.partition([oracle.vector(v["i"], v["extent"]) for v in c3["ops"]], 999), "c3")
    c4 = workloads.config(4, scale=0.02)
    print("partition config4 scaled", flush=True)
    got = parts_to_numpy(nb.nacho_partition([dcsr_operand(m) for m in c4["ops"]], 777))
    ref = oracle.partition([oracle.dcsr(m["pos0"], m["crd0"], m["pos1"], m["crd1"], m["n_rows"], m["n_cols"])
                            for m in c4["ops"]], 777)
    _compare(got, ref, "c4")
    # Theorem 1 on the GPU result: work per partition within k-1 of the ideal
    work = np.diff(got["cost"])
    ideal = np.diff([(p * int(got["cost"][-1])) // 777 for p in range(778)])
    assert np.all(np.abs(work - ideal) <= 1)


def _fused_queries(P, total, grain, scale):
    if grain > 0:
        return np.minimum(np.arange(P + 1, dtype=np.int64) * grain, total * scale) // scale
    return (np.arange(P + 1, dtype=np.int64) * total) // P


@pytest.mark.parametrize("op", ["spmv", "spmm", "spadd_vec", "spadd_dcsr"])
def test_fused_call_partition_table(op):
    """The table a fused call stores in its workspace is the oracle's Algorithm 1 on the call's queries."""
    import torch
    if op in ("spmv", "spmm"):
        A = workloads.config(2, scale=0.01)["A"] if op == "spmv" else workloads.config(5, scale=0.01)["A"]
        dt = np.float64 if op == "spmv" else np.float32
        g = csr_operand({**A, "val": A["val"].astype(dt)})
        o = [oracle.csr(A["pos"], A["crd"], A["n_rows"], A["n_cols"])]
        n = 1 if op == "spmv" else 64
        code = nb.OP_SPMV if op == "spmv" else nb.OP_SPMM
        dtc = nb.F64 if op == "spmv" else nb.F32
        for P in (0, 37):
            ws = torch.empty(nb.workspace_bytes(code, [g], dtc, 0 if op == "spmv" else n, P), dtype=torch.uint8, device="cuda")
            if op == "spmv":
                nb.nacho_spmv(g, dev(np.ones(A["n_cols"], dtype=dt)), P=P, ws=ws)
            else:
                nb.nacho_spmm(g, dev(np.ones((A["n_cols"], n), dtype=dt)), P=P, ws=ws)
            torch.cuda.synchronize()
            t = nb.workspace_parts(code, [g], dtc, ws, 0 if op == "spmv" else n, P)
            total = int(A["pos"][-1])
            qs = _fused_queries(t["P"], total, t["grain"], n)
            print(f"fused table {op} P={P} -> {t['P']} grain={t['grain']}", flush=True)
            ref = oracle.partition(o, t["P"], queries=qs)
            got = {k: v.cpu().numpy() for k, v in t.items() if k in ("coord", "posn", "cost")}
            assert np.array_equal(got["posn"].astype(np.int64), ref["posn"]), (op, P)
            assert np.array_equal(got["coord"].astype(np.int64), ref["coord"]), (op, P)
            assert np.array_equal(got["cost"], ref["cost"] * n), (op, P)
    else:
        if op == "spadd_vec":
            cfg = workloads.config(3, scale=0.02)
            g = [vector_operand(v) for v in cfg["ops"]]
            o = [oracle.vector(v["i"], v["extent"]) for v in cfg["ops"]]
            fmt, rows = "vector", 0
        else:
            cfg = workloads.config(4, scale=0.02)
            g = [dcsr_operand(m) for m in cfg["ops"]]
            o = [oracle.dcsr(m["pos0"], m["crd0"], m["pos1"], m["crd1"], m["n_rows"], m["n_cols"]) for m in cfg["ops"]]
            fmt, rows = "dcsr", sum(int(m["crd0"].shape[0]) for m in cfg["ops"])
        total = sum(x.nnz for x in g)
        for P in (0, 501):
            ws = torch.empty(nb.workspace_bytes(nb.OP_SPADD, g, nb.F32, 0, P), dtype=torch.uint8, device="cuda")
            out = nb.SparseOut(fmt, rows, total, torch.float32, "cuda")
            nb.nacho_spadd_k(g, out, P=P, ws=ws)
            torch.cuda.synchronize()
            t = nb.workspace_parts(nb.OP_SPADD, g, nb.F32, ws, 0, P)
            print(f"fused table {op} P={P} -> {t['P']}", flush=True)
            _compare({k: v.cpu().numpy() for k, v in t.items() if k in ("coord", "posn", "cost")},
                     oracle.partition(o, t["P"]), (op, P))


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_third_order_csf_random(k):
    """Three compressed levels: Algorithm 1 level by level, costs two pos arrays down at the top."""
    rng = np.random.default_rng(900 + k)
    for trial in range(5):
        shape = [(4, 5, 6), (30, 40, 50), (200, 3, 400), (2, 1000, 7), (60, 60, 60)][trial]
        cs = []
        for t in range(k):
            n = int(rng.integers(0, min(int(np.prod(shape)) // 2, 6000) + 1))
            c = random_coords(rng, shape, n)
            if trial == 1 and t > 0:
                c = cs[0].copy()                       # every coordinate tied across operands
            cs.append(c)
        g, o = [], []
        for c in cs:
            arrs = to_csf3(c)
            g.append(nb.csf3(*[dev(a) for a in arrs], shape))
            o.append(oracle.Tensor([("compressed", shape[0], arrs[0], arrs[1]), ("compressed", shape[1], arrs[2], arrs[3]),
                                    ("compressed", shape[2], arrs[4], arrs[5])]))
        total = sum(len(c) for c in cs)
        for P in (1, 2, 7, 64, 300, total + 2):
            print(f"partition csf3 k={k} trial={trial} shape={shape} total={total} P={P}", flush=True)
            got = parts_to_numpy(nb.nacho_partition(g, P))
            _compare(got, oracle.partition(o, P), (k, trial, P))


def test_third_order_csf_product_is_refused_and_its_sum_needs_three_output_levels():
    c = np.array([[0, 1, 2], [1, 0, 0]], dtype=np.int64)
    arrs = [dev(a) for a in to_csf3(c)]
    op = nb.csf3(*arrs, (2, 2, 3), dev(np.ones(2, np.float32)))
    out = nb.SparseOut("vector", 0, 4, torch.float32, "cuda")
    with pytest.raises(nb.NachoError) as e:
        nb.nacho_spadd_k([op, op], out)                 # (an output without pos0 / pos2 / crd2)
    assert e.value.status == -1
    out3 = nb.SparseOut("csf3", 4, 4, torch.float32, "cuda", cap_fibres=4)
    with pytest.raises(nb.NachoError) as e:
        nb.nacho_spmul_k([op, op], out3)
    assert e.value.status == -2
