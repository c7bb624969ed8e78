"""GPU: what the wavefronts of the executing kernels really worked on, read from the instrumented
build of the library (one record per wavefront: the items and rows it walked).

The balance claim of the method (Section 3.2.2, Theorem 1) is about these numbers: the partitions'
items add up to the total cost Q* of the iteration space, and no partition holds more than the ideal
share plus one item per further operand.  The partition test checks it on the boundaries' stored
costs; this one checks it on what the executing kernel counted while it ran."""
import numpy as np
import pytest
import torch

from paper_2604_17198_amd import binding as nb
from paper_2604_17198_amd import workloads
from gpu_util import csr_operand, dev

pytestmark = pytest.mark.gpu


def _records(fn, n_records):
    """Run `fn` once through the instrumented library and return its wavefront records."""
    rb = np.dtype(nb.WAVE_RECORD).itemsize
    nb.select_library(True)
    try:
        assert int(nb.lib().nacho_instrument_record_bytes()) == rb
        rec = torch.zeros(n_records * rb, dtype=torch.uint8, device="cuda")
        nb.instrument(rec)
        fn()
        torch.cuda.synchronize()
        nb.instrument(None)
        r = rec.cpu().numpy().view(np.dtype(nb.WAVE_RECORD))
    finally:
        nb.select_library(False)
    return r


@pytest.mark.parametrize("P", [0, 1000, 40000])
def test_spmv_wavefronts_walk_every_non_zero_once_and_within_the_bound(P):
    cfg = workloads.spmv_config(200_000, 3_000_000, 1.2, 50_000, seed=5, dtype=np.float64)
    A = cfg["A"]
    Q = int(A["pos"][-1])
    op = csr_operand(A)
    x = dev(cfg["x"])
    y = torch.empty(A["n_rows"], dtype=torch.float64, device="cuda")
    Pe = nb.num_partitions(nb.OP_SPMV, [op], nb.dtype_code(torch.float64), 0, P)
    print(f"balance spmv Q={Q} P={P} Pe={Pe}", flush=True)
    r = _records(lambda: nb.nacho_spmv(op, x, y, P=P), Pe)
    assert np.all(r["t_begin"] > 0), "a wavefront left no record"
    items = r["items"].astype(np.int64)
    assert int(items.sum()) == Q
    share = -(-Q // Pe)
    assert int(items.max()) <= share, (int(items.max()), share)       # k = 1: never above the ideal share


@pytest.mark.parametrize("k", [2, 3, 5])
def test_merge_workgroups_walk_every_entry_once_and_within_the_bound(k):
    extent = 1 << 26
    sizes = [400_000, 250_000, 900_000, 10, 123_457][:k]
    cfg = workloads.spadd_vec3_config(extent, sizes, seed=40 + k, share_frac=0.3, dtype=np.float32)
    ops = [nb.vector(dev(v["i"]), extent, dev(v["v"])) for v in cfg["ops"]]
    Q = sum(int(v["i"].shape[0]) for v in cfg["ops"])
    out = nb.SparseOut("vector", 0, Q, torch.float32, "cuda")
    Pe = nb.num_partitions(nb.OP_SPADD, ops, nb.dtype_code(torch.float32), 0, 0)
    W = nb.merge_wavefronts()
    print(f"balance merge k={k} Q={Q} Pe={Pe} wavefronts/workgroup={W}", flush=True)
    r = _records(lambda: nb.nacho_spadd_k(ops, out), Pe * W)
    assert np.all(r["t_begin"] > 0), "a wavefront left no record"
    per_wg = r["items"].astype(np.int64).reshape(Pe, W).sum(axis=1)
    assert int(per_wg.sum()) == Q
    share = -(-Q // Pe)
    assert int(per_wg.max()) <= share + k - 1, (int(per_wg.max()), share)
    assert int(out.status.cpu()[0]) == 0


def test_spmm_wavefronts_walk_every_non_zero_once():
    cfg = workloads.spmm_config(50_000, 1_000_000, 1.2, 10_000, 32, seed=9, dtype=np.float32)
    A = cfg["A"]
    Q = int(A["pos"][-1])
    op = csr_operand(A)
    B = dev(cfg["B"])
    Cout = torch.empty(A["n_rows"], 32, dtype=torch.float32, device="cuda")
    Pe = nb.num_partitions(nb.OP_SPMM, [op], nb.dtype_code(torch.float32), 32, 0)
    print(f"balance spmm Q={Q} Pe={Pe}", flush=True)
    r = _records(lambda: nb.nacho_spmm(op, B, Cout), Pe)
    assert np.all(r["t_begin"] > 0)
    items = r["items"].astype(np.int64)
    assert int(items.sum()) == Q and int(items.max()) <= -(-Q // Pe)
