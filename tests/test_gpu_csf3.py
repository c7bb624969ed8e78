"""GPU parity: nacho_spadd_k on third-order CSF tensors vs the oracle's three-level union merge.
All six level arrays and the counts must be bit-exact; values within 1e-5 (fp32) / 1e-12 (fp64) of
the oracle's double sum, relative to max(|ref|, sum of |terms|)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_17198_amd import binding as nb
from gpu_util import dev
from util import to_csf3, tol_ok

pytestmark = pytest.mark.gpu

TOL = {np.float32: 1e-5, np.float64: 1e-12}
LEVELS = ("pos0", "crd0", "pos1", "crd1", "pos2", "crd2")


def _coords(rng, shape, n):
    """About n distinct sorted coordinate triples of a tensor of `shape` (int64 [m, 3])."""
    total = int(shape[0]) * int(shape[1]) * int(shape[2])
    lin = np.unique(rng.integers(0, total, n, dtype=np.int64))
    return np.stack(np.unravel_index(lin, shape), axis=1).astype(np.int64).reshape(-1, 3)


def _tensor(coords, vals):
    d = dict(zip(LEVELS, to_csf3(coords)))
    d["val"] = vals
    return d


def _run(tens, shape, P, caps=None):
    ops = [nb.csf3(*[dev(t[n]) for n in LEVELS], shape, dev(t["val"])) for t in tens]
    cap = [sum(t[n].shape[0] for t in tens) for n in ("crd0", "crd1", "crd2")] if caps is None else caps
    out = nb.SparseOut("csf3", cap[0], cap[2], dev(tens[0]["val"]).dtype, "cuda", cap_fibres=cap[1])
    nb.nacho_spadd_k(ops, out, P=P)
    torch.cuda.synchronize()
    counts = [int(v) for v in out.counts.cpu().numpy()]
    return out, counts, int(out.status.cpu().numpy()[0])


def _check(tens, shape, P, tag):
    print(f"spadd csf3 {tag} k={len(tens)} nnz={[t['crd2'].shape[0] for t in tens]} shape={shape} P={P}", flush=True)
    out, counts, status = _run(tens, shape, P)
    ref = oracle.spadd_csf3(tens)
    n0, n1, n2 = ref["crd0"].shape[0], ref["crd1"].shape[0], ref["crd2"].shape[0]
    assert status == 0 and counts == [n0, n1, n2], (tag, status, counts, (n0, n1, n2))
    got = {n: getattr(out, n).cpu().numpy() for n in LEVELS}
    assert got["pos0"].tolist() == [0, n0], tag
    assert np.array_equal(got["crd0"][:n0], ref["crd0"]), tag
    assert np.array_equal(got["pos1"][:n0 + 1], ref["pos1"]), tag
    assert np.array_equal(got["crd1"][:n1], ref["crd1"]), tag
    assert np.array_equal(got["pos2"][:n1 + 1], ref["pos2"]), tag
    assert np.array_equal(got["crd2"][:n2], ref["crd2"]), tag
    dtype = tens[0]["val"].dtype.type
    ok = tol_ok(out.val.cpu().numpy()[:n2], ref["val"], ref["abs"], TOL[dtype])
    assert ok.all(), (tag, int((~ok).sum()))


@pytest.mark.parametrize("k", [1, 2, 3, 4, 6])
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_random_tensors(k, dtype):
    rng = np.random.default_rng(900 + k)
    shapes = [(4, 5, 6), (60, 70, 80), (3, 2000, 50), (3000, 4, 2000), (1 << 20, 1 << 10, 1 << 10)]
    for trial, shape in enumerate(shapes):
        total = shape[0] * shape[1] * shape[2]
        tens, first = [], None
        for t in range(k):
            n = int(rng.integers(0, min(total, 30000) + 1))
            c = _coords(rng, shape, n)
            if trial == 1 and t > 0:
                c = first.copy()                         # every coordinate tied
            if trial == 2 and t == 1:
                c = np.zeros((0, 3), np.int64)           # an empty operand
            if t == 0:
                first = c
            tens.append(_tensor(c, rng.uniform(-1, 1, c.shape[0]).astype(dtype)))
        for P in (0, 1, 7, 300):
            _check(tens, shape, P, f"random{trial}")


def test_long_fibres_and_long_slices_span_partitions():
    """A fibre (a slice) much longer than one partition: its head is written once, by the partition
    that holds its first entry."""
    rng = np.random.default_rng(17)
    shape = (6, 5, 1 << 20)
    tens = []
    for t in range(3):
        parts = []
        for (i, j, n) in ((1, 2, 40000), (1, 3, 25000), (4, 0, 30000), (4, 4, 9)):
            kk = np.unique(rng.integers(0, shape[2], n))
            parts.append(np.stack([np.full_like(kk, i), np.full_like(kk, j), kk], axis=1))
        c = np.concatenate(parts).astype(np.int64)
        tens.append(_tensor(c, rng.uniform(-1, 1, c.shape[0]).astype(np.float32)))
    for P in (0, 5, 64):
        _check(tens, shape, P, "long")


def test_many_partitions_cross_a_chunk_of_the_prefix_look_up():
    """More partitions than one chunk of the two-level prefix holds."""
    rng = np.random.default_rng(23)
    shape = (500, 300, 400)
    tens = []
    for t in range(2):
        c = _coords(rng, shape, 1_500_000)
        tens.append(_tensor(c, rng.uniform(-1, 1, c.shape[0]).astype(np.float32)))
    _check(tens, shape, 0, "chunks")
    _check(tens, shape, 2000, "chunks")


def test_empty_result_and_capacity():
    shape = (9, 9, 9)
    z = np.zeros((0, 3), np.int64)
    tens = [_tensor(z, np.zeros(0, np.float32)) for _ in range(2)]
    out, counts, status = _run(tens, shape, 0)
    assert status == 0 and counts == [0, 0, 0] and out.pos0.cpu().numpy().tolist() == [0, 0]
    rng = np.random.default_rng(3)
    tens = []
    for t in range(2):
        c = _coords(rng, (20, 30, 40), 6000)
        tens.append(_tensor(c, rng.uniform(-1, 1, c.shape[0]).astype(np.float32)))
    ref = oracle.spadd_csf3(tens)
    need = [ref["crd0"].shape[0], ref["crd1"].shape[0], ref["crd2"].shape[0]]
    for short in range(3):
        caps = list(need)
        caps[short] -= 1
        out, counts, status = _run(tens, (20, 30, 40), 0, caps=caps)
        assert status == -4 and counts == need, (short, status, counts, need)
    out, counts, status = _run(tens, (20, 30, 40), 0, caps=need)
    assert status == 0 and np.array_equal(out.crd2.cpu().numpy()[:need[2]], ref["crd2"])


def test_product_of_third_order_tensors_is_refused():
    rng = np.random.default_rng(4)
    c = _coords(rng, (5, 5, 5), 30)
    t = _tensor(c, np.ones(c.shape[0], np.float32))
    ops = [nb.csf3(*[dev(t[n]) for n in LEVELS], (5, 5, 5), dev(t["val"])) for _ in range(2)]
    out = nb.SparseOut("csf3", 10, 100, torch.float32, "cuda", cap_fibres=50)
    with pytest.raises(Exception):
        nb.nacho_spmul_k(ops, out)
