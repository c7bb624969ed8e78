"""Pins for the oracle's one-operand CSR partition in Python integers (operands of 2^31 entries or more;
no GPU).  Pinned to the C oracle's Algorithm 1 on operands that fit int32 (itself pinned by brute force
elsewhere), to the closed form "boundary b is the stored entry of rank Q_b in row-major order" by brute
force, and to positions beyond 2^31 built so that the answer is known in closed form."""
import numpy as np
import pytest

import oracle
from util import random_coords, to_csr


def _rows(pos, crd):
    return lambda r: crd[pos[r]:pos[r + 1]]


@pytest.mark.parametrize("seed", range(6))
def test_equals_the_c_oracle_and_the_rank_q_entry(seed):
    rng = np.random.default_rng(40 + seed)
    n_rows, n_cols = int(rng.integers(1, 60)), int(rng.integers(1, 60))
    nnz = int(rng.integers(0, n_rows * n_cols // 2 + 1))
    c = random_coords(rng, (n_rows, n_cols), nnz)
    if seed % 2 == 0 and nnz:                      # runs of empty rows
        c = c[c[:, 0] % 3 != 1]
    pos, crd = to_csr(c, n_rows)
    for P in (1, 2, 7, max(1, c.shape[0]), c.shape[0] + 5):
        got = oracle.partition_csr64(pos.astype(np.int64), _rows(pos, crd), n_cols, P)
        ref = oracle.partition([oracle.csr(pos, crd, n_rows, n_cols)], P)
        assert np.array_equal(got["coord"], ref["coord"]), (seed, P)
        assert np.array_equal(got["posn"], ref["posn"][:, 0, :]), (seed, P)
        assert np.array_equal(got["cost"], ref["cost"]), (seed, P)
        total = c.shape[0]
        for p in range(1, P):
            Q = p * total // P
            if Q < total:                          # the entry of rank Q in row-major order
                assert tuple(got["coord"][p]) == tuple(int(v) for v in c[Q]), (seed, P, p)
                assert got["posn"][p, 1] == Q and got["cost"][p] == Q


def test_positions_beyond_32_bits():
    """Every row holds the columns 0 .. L-1: the entry of rank Q is (Q // L, Q % L), whatever the size."""
    L, n_rows = 3_000_000, 1000                    # 3e9 entries, none of them stored
    pos = np.arange(n_rows + 1, dtype=np.int64) * L
    assert pos[-1] > 2**31
    row = lambda r: np.arange(L, dtype=np.int64)
    P = 37
    got = oracle.partition_csr64(pos, row, L, P)
    for p in range(1, P):
        Q = p * int(pos[-1]) // P
        assert tuple(got["coord"][p]) == (Q // L, Q % L) and got["posn"][p, 1] == Q and got["cost"][p] == Q
    assert tuple(got["coord"][P]) == (n_rows, 0) and got["posn"][P, 1] == pos[-1] and got["cost"][P] == pos[-1]
