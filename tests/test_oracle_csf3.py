"""Pins for the oracle's union addition of third-order CSF tensors (no GPU).

The oracle walks the three-level coiteration nest (Section 2.2's nest, one level deeper).  Pinned to
the plain definition by other means: dense evaluation (numpy scatter-add into a dense cube; the stored
pattern of the result is the union of the operands' stored patterns), numpy.unique on linearised
coordinates, the level arrays rebuilt from the sorted coordinate list by an independent routine, and
the two-level addition on the same data with the two leading modes fused.
"""
import numpy as np
import pytest

import oracle
from util import random_coords, to_csf3, to_dcsr


def _tensor(coords, vals):
    p0, c0, p1, c1, p2, c2 = to_csf3(coords)
    return {"pos0": p0, "crd0": c0, "pos1": p1, "crd1": c1, "pos2": p2, "crd2": c2, "val": vals}


def _expand(t):
    """Coordinate triples of a CSF tensor, in storage order."""
    out = []
    for a in range(t["pos0"][0], t["pos0"][1]):
        for b in range(t["pos1"][a], t["pos1"][a + 1]):
            for c in range(t["pos2"][b], t["pos2"][b + 1]):
                out.append((int(t["crd0"][a]), int(t["crd1"][b]), int(t["crd2"][c])))
    return out


@pytest.mark.parametrize("k", [1, 2, 3, 5])
def test_against_dense_evaluation(k):
    rng = np.random.default_rng(300 + k)
    shape = (4, 5, 6)
    for trial in range(20):
        lists = [random_coords(rng, shape, int(rng.integers(0, 40))) for _ in range(k)]
        if trial % 4 == 1 and k > 1:
            lists[1] = lists[0].copy()
        vals = [rng.uniform(-1, 1, c.shape[0]) for c in lists]
        dense = np.zeros(shape)
        stored = np.zeros(shape, dtype=bool)
        for c, v in zip(lists, vals):
            np.add.at(dense, tuple(c.T), v)
            stored[tuple(c.T)] = True
        r = oracle.spadd_csf3([_tensor(c, v) for c, v in zip(lists, vals)])
        coords = _expand(r)
        want = [tuple(int(x) for x in c) for c in np.argwhere(stored)]        # argwhere: lexicographic order
        assert coords == want, (k, trial)
        assert np.allclose(r["val"], [dense[c] for c in want], rtol=0, atol=1e-14)
        # the level arrays are those of the sorted coordinate list
        ref = to_csf3(np.array(want, dtype=np.int64).reshape(-1, 3))
        for name, arr in zip(("pos0", "crd0", "pos1", "crd1", "pos2", "crd2"), ref):
            assert np.array_equal(r[name], arr), (k, trial, name)


def test_against_unique_of_linearised_coordinates_and_value_order():
    rng = np.random.default_rng(7)
    shape = (30, 20, 25)
    lists = [random_coords(rng, shape, n) for n in (700, 300, 900)]
    lists[2][:200] = lists[0][:200]                                             # forced coincidences
    lists[2] = np.unique(lists[2], axis=0)
    vals = [rng.uniform(-1, 1, c.shape[0]).astype(np.float32) for c in lists]
    r = oracle.spadd_csf3([_tensor(c, v) for c, v in zip(lists, vals)])
    lin = lambda c: (c[:, 0] * shape[1] + c[:, 1]) * shape[2] + c[:, 2]
    allc = np.unique(np.concatenate([lin(c) for c in lists]))
    got = np.array(_expand(r), dtype=np.int64)
    assert np.array_equal(lin(got), allc)
    # values: operand order, in double
    acc = {}
    for c, v in zip(lists, vals):
        for key, x in zip(lin(c).tolist(), v.tolist()):
            acc[key] = acc.get(key, 0.0) + float(x)
    assert np.array_equal(r["val"], np.array([acc[key] for key in allc.tolist()]))


def test_fused_leading_modes_equal_the_dcsr_addition():
    """(i, j, k) with i and j fused into one mode is a DCSR matrix: same entries, same values."""
    rng = np.random.default_rng(9)
    shape = (7, 9, 11)
    lists = [random_coords(rng, shape, n) for n in (120, 80)]
    vals = [rng.uniform(-1, 1, c.shape[0]) for c in lists]
    r3 = oracle.spadd_csf3([_tensor(c, v) for c, v in zip(lists, vals)])
    mats = []
    for c, v in zip(lists, vals):
        fused = np.stack([c[:, 0] * shape[1] + c[:, 1], c[:, 2]], 1)
        p0, c0, p1, c1 = to_dcsr(fused)
        mats.append({"pos0": p0, "crd0": c0, "pos1": p1, "crd1": c1, "val": v})
    r2 = oracle.spadd_dcsr(mats)
    assert np.array_equal(r3["crd2"], r2["crd1"]) and np.array_equal(r3["val"], r2["val"])
    assert np.array_equal(r3["pos2"], r2["pos1"])
    fused_rows = r3["crd0"][np.searchsorted(r3["pos1"], np.arange(r3["crd1"].shape[0]), side="right") - 1] \
        * shape[1] + r3["crd1"]
    assert np.array_equal(fused_rows, r2["crd0"])


def test_empty_operands_and_empty_result():
    z = _tensor(np.zeros((0, 3), np.int64), np.zeros(0))
    r = oracle.spadd_csf3([z, z])
    assert r["pos0"].tolist() == [0, 0] and r["crd2"].shape[0] == 0 and r["pos1"].tolist() == [0]
    one = _tensor(np.array([[2, 3, 4]]), np.array([0.5]))
    r = oracle.spadd_csf3([z, one, z])
    assert _expand(r) == [(2, 3, 4)] and r["val"].tolist() == [0.5]


def test_generated_benchmark_tensors_are_valid_csf_and_add_up():
    """The seeded CSF generator the benchmark uses: its level arrays equal those rebuilt from its own
    coordinate list, and the oracle's sum of two of its tensors matches numpy.unique."""
    from paper_2604_17198_amd import workloads
    shape = (20, 30, 40)
    cfg = workloads.csf3_add_config(k=2, shape=shape, nnz_each=3000, seed=5)
    names = ("pos0", "crd0", "pos1", "crd1", "pos2", "crd2")
    for t in cfg["ops"]:
        coords = np.stack(np.unravel_index(t["lin"], shape), axis=1)
        for n, a in zip(names, to_csf3(coords)):
            assert np.array_equal(t[n], a), n
    r = oracle.spadd_csf3(cfg["ops"])
    union = np.unique(np.concatenate([t["lin"] for t in cfg["ops"]]))
    got = np.array(_expand(r), dtype=np.int64)
    assert np.array_equal((got[:, 0] * shape[1] + got[:, 1]) * shape[2] + got[:, 2], union)
    shared = np.intersect1d(cfg["ops"][0]["lin"], cfg["ops"][1]["lin"]).shape[0]
    assert shared >= 0.15 * 3000                       # the forced coincidences are there
