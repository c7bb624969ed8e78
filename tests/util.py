"""Test helpers: tiny random sparse tensors built from explicit coordinate sets,
and brute-force references written straight from definitions (sorted lists,
dense arrays).  Nothing here is shared with the oracle or the HIP library."""
from __future__ import annotations

import numpy as np


def random_coords(rng, shape, nnz):
    """`nnz` distinct coordinate tuples of a tensor of `shape`, sorted
    lexicographically (array [n, d])."""
    total = int(np.prod(shape))
    nnz = min(nnz, total)
    flat = np.sort(rng.choice(total, size=nnz, replace=False))
    return np.stack(np.unravel_index(flat, shape), axis=1).astype(np.int64).reshape(nnz, len(shape))


def to_vector(coords):
    return coords[:, 0].astype(np.int32)


def to_csr(coords, n_rows):
    counts = np.bincount(coords[:, 0], minlength=n_rows)
    pos = np.zeros(n_rows + 1, dtype=np.int32)
    pos[1:] = np.cumsum(counts)
    return pos, coords[:, 1].astype(np.int32)


def to_dcsr(coords):
    if coords.shape[0] == 0:
        return (np.array([0, 0], np.int32), np.zeros(0, np.int32),
                np.array([0], np.int32), np.zeros(0, np.int32))
    rows, counts = np.unique(coords[:, 0], return_counts=True)
    pos1 = np.zeros(rows.shape[0] + 1, dtype=np.int32)
    pos1[1:] = np.cumsum(counts)
    return (np.array([0, rows.shape[0]], np.int32), rows.astype(np.int32),
            pos1, coords[:, 1].astype(np.int32))


def to_csf3(coords):
    """Three compressed levels (pos0, crd0, pos1, crd1, pos2, crd2)."""
    if coords.shape[0] == 0:
        z = np.zeros(0, np.int32)
        return (np.array([0, 0], np.int32), z, np.array([0], np.int32), z, np.array([0], np.int32), z)
    i_u, i_first = np.unique(coords[:, 0], return_index=True)
    ij = coords[:, :2]
    change = np.ones(coords.shape[0], dtype=bool)
    change[1:] = np.any(ij[1:] != ij[:-1], axis=1)
    ij_first = np.flatnonzero(change)
    crd1 = coords[ij_first, 1]
    # pos1: for each i, range of (i,j) fibres
    pos1 = np.searchsorted(ij_first, np.append(i_first, coords.shape[0])).astype(np.int32)
    pos2 = np.append(ij_first, coords.shape[0]).astype(np.int32)
    return (np.array([0, i_u.shape[0]], np.int32), i_u.astype(np.int32), pos1,
            crd1.astype(np.int32), pos2, coords[:, 2].astype(np.int32))


def lex_less(a, b):
    """a < b for coordinate tuples (python tuples compare lexicographically)."""
    return tuple(int(v) for v in a) < tuple(int(v) for v in b)


def merged_sorted(coord_lists):
    """All stored coordinate tuples of all operands, sorted (duplicates kept)."""
    allc = [tuple(int(v) for v in c) for cl in coord_lists for c in cl]
    return sorted(allc)


def count_prefix_less(coords, m, boundary):
    """Number of distinct level-m entries (coordinate prefixes of length m+1)
    of one operand that are lexicographically before boundary[:m+1]."""
    pre = sorted({tuple(int(v) for v in c[:m + 1]) for c in coords})
    b = tuple(int(v) for v in boundary[:m + 1])
    return sum(1 for p in pre if p < b)


def tol_ok(got, ref, sabs, tol):
    """|got - ref| <= tol * max(|ref|, sum|terms|), elementwise."""
    got = np.asarray(got, dtype=np.float64)
    return np.abs(got - ref) <= tol * np.maximum(np.abs(ref), sabs)
