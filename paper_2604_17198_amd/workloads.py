"""Seeded synthetic inputs for the five benchmark configurations.

This module only *generates data* (numpy, host memory).  It holds none of the
partitioning or kernel arithmetic: both the CPU oracle's tests and the HIP
path's tests/bench feed on the arrays produced here, and neither the oracle nor
the HIP library imports it.

The paper evaluates on SuiteSparse / FROSTT tensors and on unpublished
"synthetic power-law matrices" (Evaluation, skew experiment).  None of those
is available, so the generators below stand in for them: they reproduce the
workload *structure* (power-law row skew, hyper-sparse rows, partially
overlapping operand pairs), not any record of those suites.

Row lengths follow the rank-frequency form of Zipf's law,
    L_r = clip(floor(C * r**(-alpha)), 1, cap),   r = 1..n_nonempty,
with C solved by bisection so that sum(L_r) hits the requested nnz; ranks are
assigned to rows by a random permutation and the empty rows are chosen
uniformly.  (Sampling lengths i.i.d. from a Zipf law cannot meet a requested
nnz total, a cap and an empty-row fraction at the same time.)
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "zipf_row_lengths", "csr_powerlaw", "dcsr_powerlaw", "sparse_vector",
    "spmv_config", "spadd_vec3_config", "spadd_dcsr_config", "spmm_config", "csr_add_config",
    "config", "CONFIG_NAMES",
]

CONFIG_NAMES = {
    1: "C1 SpMV fp64 4096x4096 ~40k nnz Zipf(1.5)",
    2: "C2 SpMV fp64 2Mx2M ~50M nnz Zipf(1.3)",
    3: "C3 3-way sparse-vector add fp32 2^30, 10M+1M+100k nnz",
    4: "C4 DCSR A+B fp32 1Mx1M 2x~20M nnz Zipf(1.4)",
    5: "C5 SpMM fp32 A 1Mx1M ~30M nnz Zipf(1.3) x B 1Mx64",
}


# --------------------------------------------------------------------------- #
# row-length law
# --------------------------------------------------------------------------- #
def zipf_row_lengths(n_nonempty: int, alpha: float, cap: int, target_nnz: int) -> np.ndarray:
    """Lengths by rank (descending), each in [1, cap], summing to ~target_nnz."""
    if n_nonempty <= 0:
        return np.zeros(0, dtype=np.int64)
    r = np.arange(1, n_nonempty + 1, dtype=np.float64)
    w = r ** (-alpha)

    def total(c: float) -> int:
        return int(np.clip(np.floor(c * w), 1, cap).sum())

    lo, hi = 0.0, 1.0
    while total(hi) < target_nnz and hi < 1e18:
        hi *= 2.0
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if total(mid) < target_nnz:
            lo = mid
        else:
            hi = mid
        if hi - lo <= 1e-9 * hi:
            break
    return np.clip(np.floor(hi * w), 1, cap).astype(np.int64)


def _sorted_unique_columns(rng, rows: np.ndarray, lengths: np.ndarray, n_cols: int):
    """For every (row, length) draw `length` column indices, uniform without
    replacement, sorted.  Rows with length >= n_cols/16 use a permutation
    prefix (exact length); lighter rows draw with replacement and drop the few
    duplicates.  `rows` must be strictly increasing.  Returns (counts, cols)."""
    heavy = lengths >= max(1, n_cols // 16)
    light = ~heavy
    keys = []
    if light.any():
        lr = rows[light].astype(np.int64)
        ll = lengths[light]
        rep = np.repeat(lr, ll)
        cols = rng.integers(0, n_cols, size=rep.shape[0], dtype=np.int64)
        keys.append(rep * n_cols + cols)
        del rep, cols
    for r, L in zip(rows[heavy].tolist(), lengths[heavy].tolist()):
        L = min(int(L), n_cols)
        cols = rng.permutation(n_cols)[:L].astype(np.int64)
        keys.append(r * n_cols + cols)
    if not keys:
        return np.zeros(rows.shape[0], dtype=np.int64), np.zeros(0, dtype=np.int32)
    key = np.concatenate(keys) if len(keys) > 1 else keys[0]
    del keys
    key.sort(kind="stable")
    if key.shape[0] > 1:
        keep = np.empty(key.shape[0], dtype=bool)
        keep[0] = True
        np.not_equal(key[1:], key[:-1], out=keep[1:])
        key = key[keep]
    krow = key // n_cols
    cols = (key - krow * n_cols).astype(np.int32)
    # counts per listed row (rows are sorted, so searchsorted maps row id -> slot)
    slot = np.searchsorted(rows, krow)
    counts = np.bincount(slot, minlength=rows.shape[0]).astype(np.int64)
    return counts, cols


def _uniform_values(rng, n: int, dtype) -> np.ndarray:
    return rng.uniform(-1.0, 1.0, size=n).astype(dtype)


# --------------------------------------------------------------------------- #
# formats
# --------------------------------------------------------------------------- #
def csr_powerlaw(n_rows, n_cols, target_nnz, alpha, cap, empty_frac, seed, dtype):
    """CSR (dense rows, compressed columns) with power-law row lengths.
    Returns dict(pos int32[n_rows+1], crd int32[nnz], val dtype[nnz])."""
    rng = np.random.default_rng(seed)
    n_nonempty = int(round(n_rows * (1.0 - empty_frac)))
    lengths = zipf_row_lengths(n_nonempty, alpha, min(cap, n_cols), target_nnz)
    rows = np.sort(rng.choice(n_rows, size=n_nonempty, replace=False)) if n_nonempty < n_rows \
        else np.arange(n_rows, dtype=np.int64)
    lengths = lengths[rng.permutation(n_nonempty)]          # rank -> row at random
    counts, crd = _sorted_unique_columns(rng, rows, lengths, n_cols)
    per_row = np.zeros(n_rows, dtype=np.int64)
    per_row[rows] = counts
    pos = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(per_row, out=pos[1:])
    assert pos[-1] == crd.shape[0] and pos[-1] < 2**31
    return {"n_rows": int(n_rows), "n_cols": int(n_cols),
            "pos": pos.astype(np.int32), "crd": crd,
            "val": _uniform_values(rng, crd.shape[0], dtype)}


def dcsr_powerlaw(n_rows, n_cols, target_nnz, alpha, cap, stored_rows, seed, dtype):
    """DCSR (compressed rows, compressed columns); `stored_rows` is the sorted
    array of non-empty row ids.  Returns dict(pos0 int32[2], crd0 int32[nr],
    pos1 int32[nr+1], crd1 int32[nnz], val dtype[nnz])."""
    rng = np.random.default_rng(seed)
    rows = np.asarray(stored_rows, dtype=np.int64)
    nr = rows.shape[0]
    lengths = zipf_row_lengths(nr, alpha, min(cap, n_cols), target_nnz)
    lengths = lengths[rng.permutation(nr)]
    counts, crd1 = _sorted_unique_columns(rng, rows, lengths, n_cols)
    keep = counts > 0                                      # a stored row holds >= 1 entry
    rows, counts = rows[keep], counts[keep]
    pos1 = np.zeros(rows.shape[0] + 1, dtype=np.int64)
    np.cumsum(counts, out=pos1[1:])
    assert pos1[-1] == crd1.shape[0] and pos1[-1] < 2**31
    return {"n_rows": int(n_rows), "n_cols": int(n_cols),
            "pos0": np.array([0, rows.shape[0]], dtype=np.int32),
            "crd0": rows.astype(np.int32), "pos1": pos1.astype(np.int32),
            "crd1": crd1, "val": _uniform_values(rng, crd1.shape[0], dtype)}


def _sorted_unique_indices(rng, n: int, extent: int) -> np.ndarray:
    """n sorted unique integers, uniform over [0, extent)."""
    if n >= extent:
        return np.arange(extent, dtype=np.int64)
    if n * 4 >= extent:
        return np.sort(rng.choice(extent, size=n, replace=False)).astype(np.int64)
    got = np.unique(rng.integers(0, extent, size=int(n * 1.02) + 16, dtype=np.int64))
    while got.shape[0] < n:
        more = rng.integers(0, extent, size=n - got.shape[0] + 16, dtype=np.int64)
        got = np.unique(np.concatenate([got, more]))
    if got.shape[0] > n:
        got = got[np.sort(rng.choice(got.shape[0], size=n, replace=False))]
    return got


def sparse_vector(n, extent, seed, dtype, share_from=None, share_frac=0.0):
    """Sparse vector: sorted unique int32 indices `i` and values `v`.  A
    fraction `share_frac` of the indices is drawn (without replacement) from
    `share_from`, the rest uniformly from [0, extent)."""
    rng = np.random.default_rng(seed)
    n_shared = 0
    parts = []
    if share_from is not None and share_frac > 0 and share_from.shape[0] > 0:
        n_shared = min(int(round(n * share_frac)), share_from.shape[0])
        pick = rng.choice(share_from.shape[0], size=n_shared, replace=False)
        parts.append(np.asarray(share_from, dtype=np.int64)[pick])
    parts.append(_sorted_unique_indices(rng, n - n_shared, extent))
    idx = np.unique(np.concatenate(parts))
    return {"extent": int(extent), "i": idx.astype(np.int32),
            "v": _uniform_values(rng, idx.shape[0], dtype)}


def csf3_tensor(shape, nnz, seed, dtype, share_from=None, share_frac=0.0):
    """Third-order tensor with three compressed levels (CSF): `nnz` distinct coordinates uniform over
    `shape`, a fraction `share_frac` of them taken from the linearised coordinates `share_from` of
    another tensor.  Returns the six level arrays (int32), the values and `lin`, the sorted linearised
    coordinates (i * J + j) * K + k."""
    rng = np.random.default_rng(seed)
    I, J, K = (int(v) for v in shape)
    parts, n_shared = [], 0
    if share_from is not None and share_frac > 0 and share_from.shape[0] > 0:
        n_shared = min(int(round(nnz * share_frac)), share_from.shape[0])
        parts.append(share_from[rng.choice(share_from.shape[0], size=n_shared, replace=False)])
    parts.append(_sorted_unique_indices(rng, nnz - n_shared, I * J * K))
    lin = np.unique(np.concatenate(parts))
    i, rest = np.divmod(lin, J * K)
    j, k = np.divmod(rest, K)
    n = lin.shape[0]
    ij = i * J + j
    fibre_first = np.flatnonzero(np.concatenate([[True], ij[1:] != ij[:-1]])) if n else np.zeros(0, np.int64)
    fi = i[fibre_first]                                         # slice of every fibre
    slice_first = np.flatnonzero(np.concatenate([[True], fi[1:] != fi[:-1]])) if n else np.zeros(0, np.int64)
    i32 = lambda a: np.ascontiguousarray(a, dtype=np.int32)
    return {"shape": (I, J, K), "lin": lin,
            "pos0": i32([0, slice_first.shape[0]]), "crd0": i32(fi[slice_first]),
            "pos1": i32(np.append(slice_first, fibre_first.shape[0])), "crd1": i32(j[fibre_first]),
            "pos2": i32(np.append(fibre_first, n)), "crd2": i32(k),
            "val": _uniform_values(rng, n, dtype)}


def csf3_add_config(k=2, shape=(2000, 2000, 2000), nnz_each=8_000_000, seed=71, share_frac=0.2, dtype=np.float32):
    """k third-order CSF tensors of one shape for the k-way tensor addition (the shape of the paper's
    FROSTT-style operands: a few thousand coordinates per mode, millions of non-zeros; 20 % of the later
    operands' coordinates coincide with the first one's)."""
    a = csf3_tensor(shape, nnz_each, seed, dtype)
    ops = [a]
    for t in range(1, k):
        ops.append(csf3_tensor(shape, nnz_each, seed + 7919 * t, dtype, share_from=a["lin"], share_frac=share_frac))
    return {"kind": "spadd_csf3", "ops": ops, "shape": tuple(int(v) for v in shape)}


# --------------------------------------------------------------------------- #
# the five configurations (scale < 1 shrinks sizes for CPU-side tests)
# --------------------------------------------------------------------------- #
def spmv_config(n, nnz, alpha, cap, seed, empty_frac=0.30, dtype=np.float64):
    A = csr_powerlaw(n, n, nnz, alpha, cap, empty_frac, seed, dtype)
    rng = np.random.default_rng(seed + 1000003)
    return {"kind": "spmv", "A": A, "x": _uniform_values(rng, n, dtype)}


def spadd_vec3_config(extent, sizes, seed, share_frac=0.20, dtype=np.float32):
    a = sparse_vector(sizes[0], extent, seed, dtype)
    ops = [a]
    for t, n in enumerate(sizes[1:], start=1):
        ops.append(sparse_vector(n, extent, seed + 7919 * t, dtype,
                                 share_from=a["i"], share_frac=share_frac))
    return {"kind": "spadd_vec", "ops": ops, "extent": int(extent)}


def spadd_dcsr_config(n, nnz_each, alpha, cap, stored_frac, shared_frac, seed, dtype=np.float32):
    rng = np.random.default_rng(seed)
    nr = max(1, int(round(n * stored_frac)))
    rows_a = np.sort(rng.choice(n, size=nr, replace=False))
    n_sh = int(round(nr * shared_frac))
    shared = rng.choice(rows_a, size=n_sh, replace=False)
    mask = np.ones(n, dtype=bool)
    mask[rows_a] = False
    complement = np.flatnonzero(mask)
    fresh = rng.choice(complement, size=min(nr - n_sh, complement.shape[0]), replace=False)
    rows_b = np.sort(np.concatenate([shared, fresh]))
    A = dcsr_powerlaw(n, n, nnz_each, alpha, cap, rows_a, seed + 11, dtype)
    B = dcsr_powerlaw(n, n, nnz_each, alpha, cap, rows_b, seed + 23, dtype)
    return {"kind": "spadd_dcsr", "ops": [A, B], "n_rows": int(n), "n_cols": int(n)}


def spmm_config(n, nnz, alpha, cap, n_dense, seed, dtype=np.float32):
    A = csr_powerlaw(n, n, nnz, alpha, cap, 0.0, seed, dtype)
    rng = np.random.default_rng(seed + 1000003)
    B = rng.uniform(-1.0, 1.0, size=(n, n_dense)).astype(dtype)
    return {"kind": "spmm", "A": A, "B": B, "n_dense": int(n_dense)}


def csr_add_config(k, n=100_000, nnz_each=5_000_000, alpha=1.3, seed=61, dtype=np.float32):
    """k power-law CSR matrices of one shape for the fused k-way CSR addition: the shape of the paper's skew
    experiment (synthetic power-law matrices of 100000 x 100000, Evaluation) with independent operands."""
    ops = [csr_powerlaw(n, n, nnz_each, alpha, max(8, n // 4), 0.0, seed + t, dtype) for t in range(k)]
    return {"kind": "spadd_csr", "ops": ops, "n_rows": int(n), "n_cols": int(n)}


def config(which: int, scale: float = 1.0, seed: int | None = None):
    """Inputs of configuration `which` (1..5).  `scale` multiplies the sizes
    (rows, nnz, index space) so that the CPU suite can run the same recipe
    small; scale=1 is the full-size configuration.  Seeds default to the
    configuration number."""
    s = which if seed is None else seed
    sc = float(scale)
    if which == 1:
        n = max(8, int(4096 * sc))
        return spmv_config(n, max(8, int(40_000 * sc)), 1.5, n, s)
    if which == 2:
        n = max(64, int(2_000_000 * sc))
        return spmv_config(n, max(64, int(50_000_000 * sc)), 1.3, max(8, int(1_000_000 * sc)), s)
    if which == 3:
        extent = max(1 << 12, int((1 << 30) * sc))
        sizes = [max(4, int(v * sc)) for v in (10_000_000, 1_000_000, 100_000)]
        return spadd_vec3_config(extent, sizes, s)
    if which == 4:
        n = max(64, int(1_000_000 * sc))
        return spadd_dcsr_config(n, max(64, int(20_000_000 * sc)), 1.4, max(8, n // 4), 0.10, 0.50, s)
    if which == 5:
        n = max(64, int(1_000_000 * sc))
        return spmm_config(n, max(64, int(30_000_000 * sc)), 1.3, max(8, n // 4), 64, s)
    raise ValueError(f"unknown configuration {which}")
