"""nacho_validate: the device-side check of the operands' preconditions flags planted violations
(unsorted or repeated coordinates, coordinates outside the extent, broken pos arrays) and passes
well-formed operands of every format."""
import numpy as np
import pytest
import torch

from paper_2604_17198_amd import binding as nb
from gpu_util import dev
from util import random_coords, to_csr, to_csf3, to_dcsr, to_vector

pytestmark = pytest.mark.gpu


def _ops(rng):
    shape = (300, 200)
    c = random_coords(rng, shape, 5000)
    pos, crd = to_csr(c, shape[0])
    p0, c0, p1, c1 = to_dcsr(c)
    v = to_vector(random_coords(rng, (10000,), 3000))
    c3 = random_coords(rng, (20, 30, 40), 4000)
    return {
        "vector": (lambda a: nb.vector(dev(a[0]), 10000), [v]),
        "csr": (lambda a: nb.csr(dev(a[0]), dev(a[1]), *shape), [pos, crd]),
        "dcsr": (lambda a: nb.dcsr(dev(a[0]), dev(a[1]), dev(a[2]), dev(a[3]), *shape), [p0, c0, p1, c1]),
        "coo": (lambda a: nb.coo(dev(a[0]), dev(a[1]), *shape), [c[:, 0].astype(np.int32), c[:, 1].astype(np.int32)]),
        "csf3": (lambda a: nb.csf3(*[dev(x) for x in a], (20, 30, 40)), list(to_csf3(c3))),
    }


def test_well_formed_operands_pass():
    rng = np.random.default_rng(1)
    for name, (make, arrs) in _ops(rng).items():
        status, info = nb.nacho_validate([make(arrs), make(arrs)])
        assert status == 0 and info == (-1, -1, -1), name


@pytest.mark.parametrize("name,which,how", [
    ("vector", 0, "swap"), ("vector", 0, "repeat"), ("vector", 0, "range"),
    ("csr", 1, "swap"), ("csr", 1, "range"), ("csr", 0, "pos_decreases"), ("csr", 0, "pos_end"),
    ("dcsr", 1, "repeat"), ("dcsr", 3, "swap"), ("dcsr", 2, "pos_decreases"),
    ("coo", 0, "swap_rows"), ("coo", 1, "repeat_pair"),
    ("csf3", 5, "swap"), ("csf3", 2, "pos_end"),
])
def test_planted_violations_are_flagged(name, which, how):
    rng = np.random.default_rng(2)
    make, arrs = _ops(rng)[name]
    arrs = [a.copy() for a in arrs]
    a = arrs[which]
    if how in ("swap", "swap_rows"):
        # two neighbouring coordinates of one segment out of order (a segment longer than one)
        if name == "vector" or name == "coo":
            q = 100
            if how == "swap_rows":
                q = int(np.flatnonzero(np.diff(a) > 0)[5]) + 1      # a place where the row changes
            a[q - 1], a[q] = a[q] + 1 if a[q] == a[q - 1] else a[q], a[q - 1]
        else:
            pos = arrs[which - 1]
            seg = int(np.flatnonzero(np.diff(pos) >= 2)[3])
            q = int(pos[seg]) + 1
            a[q - 1], a[q] = a[q], a[q - 1]
    elif how == "repeat":
        if name == "vector":
            a[50] = a[49]
        else:                                   # dcsr level 0: a stored row twice
            a[7] = a[6]
    elif how == "repeat_pair":
        rows = arrs[0]
        q = int(np.flatnonzero(np.diff(rows) == 0)[10]) + 1         # same row as its predecessor
        a[q] = a[q - 1]
    elif how == "range":
        a[-1] = 10**9
    elif how == "pos_decreases":
        i = len(a) // 2
        a[i] = a[i - 1] - 1 if a[i - 1] > 0 else a[i + 1] + 1
    elif how == "pos_end":
        a[-1] += 1
    status, info = nb.nacho_validate([make(arrs)])
    assert status == -1, (name, how)
    assert info[0] == 0 and info[1] >= 0 and info[2] >= 0
