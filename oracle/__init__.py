"""CPU oracle -- TEST INFRASTRUCTURE ONLY.

numpy-facing wrapper over `nacho_oracle.c` (plain serial C, compiled with gcc).
Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package; the HIP library and its Python binding never do, and this package
imports nothing from them.

Every function cites the passage of the paper it follows in the C source.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nacho_oracle.c")
_LIB = os.path.join(_HERE, "libnacho_oracle.so")

DENSE, COMPRESSED, NONUNIQUE, SINGLETON = 0, 1, 2, 3
MAXL = 3


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no GPU toolchain involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".{os.getpid()}.tmp"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def time_spmv_native(pos, crd, val, x, reps=3):
    """Benchmarks only: the same source compiled for THIS host (-O3 -march=native, into a temporary
    file: the library that travels with the tree must run on any host) and timed in C with the
    monotonic clock; returns (best seconds of `reps` runs of the fp64 SpMV, y, s)."""
    import tempfile
    path = os.path.join(tempfile.gettempdir(), f"libnacho_oracle_native_{os.getpid()}.so")
    subprocess.check_call(["gcc", "-O3", "-march=native", "-std=c11", "-fPIC", "-shared", "-o", path, _SRC, "-lm"])
    nat = C.CDLL(path)
    nat.ora_time_spmv_f64.restype = C.c_double
    pos, crd = _i32(pos), _i32(crd)
    val = np.ascontiguousarray(val, dtype=np.float64)
    x = np.ascontiguousarray(x, dtype=np.float64)
    n_rows = pos.shape[0] - 1
    y = np.zeros(n_rows, dtype=np.float64)
    s = np.zeros(n_rows, dtype=np.float64)
    best = nat.ora_time_spmv_f64(C.c_int64(n_rows), pos.ctypes.data_as(C.c_void_p), crd.ctypes.data_as(C.c_void_p),
                                 val.ctypes.data_as(C.c_void_p), x.ctypes.data_as(C.c_void_p),
                                 y.ctypes.data_as(C.c_void_p), s.ctypes.data_as(C.c_void_p), C.c_int32(reps))
    os.remove(path)
    return float(best), y, s


class _Level(C.Structure):
    _fields_ = [("kind", C.c_int32), ("extent", C.c_int64),
                ("pos", C.c_void_p), ("crd", C.c_void_p)]


class _Tensor(C.Structure):
    _fields_ = [("nlevels", C.c_int32), ("lvl", _Level * MAXL)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.ora_total_cost.restype = C.c_int64
        _lib.ora_spadd_vec.restype = C.c_int64
        _lib.ora_spadd_csr.restype = C.c_int64
        _lib.ora_spmul_vec.restype = C.c_int64
        _lib.ora_spmul_csr.restype = C.c_int64
        _lib.ora_spadd_coo.restype = C.c_int64
        _lib.ora_spmul_coo.restype = C.c_int64
    return _lib


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a


class Tensor:
    """Sparse operand as a list of levels: ("dense", N) or ("compressed", N, pos, crd)."""

    def __init__(self, levels):
        self.levels = []
        self._keep = []
        t = _Tensor()
        t.nlevels = len(levels)
        for m, l in enumerate(levels):
            if l[0] == "dense":
                t.lvl[m].kind, t.lvl[m].extent = DENSE, int(l[1])
                t.lvl[m].pos = None
                t.lvl[m].crd = None
            elif l[0] == "singleton":
                crd = _i32(l[2])
                self._keep += [crd]
                t.lvl[m].kind, t.lvl[m].extent = SINGLETON, int(l[1])
                t.lvl[m].pos = None
                t.lvl[m].crd = crd.ctypes.data
            else:
                pos, crd = _i32(l[2]), _i32(l[3])
                self._keep += [pos, crd]
                t.lvl[m].kind = NONUNIQUE if l[0] == "nonunique" else COMPRESSED
                t.lvl[m].extent = int(l[1])
                t.lvl[m].pos = pos.ctypes.data
                t.lvl[m].crd = crd.ctypes.data
        self.c = t
        self.nlevels = len(levels)


def vector(idx, extent):
    idx = _i32(idx)
    return Tensor([("compressed", extent, np.array([0, idx.shape[0]], dtype=np.int32), idx)])


def csr(pos, crd, n_rows, n_cols):
    return Tensor([("dense", n_rows), ("compressed", n_cols, pos, crd)])


def dcsr(pos0, crd0, pos1, crd1, n_rows, n_cols):
    return Tensor([("compressed", n_rows, pos0, crd0), ("compressed", n_cols, pos1, crd1)])


def coo(rows, cols, n_rows, n_cols):
    """Coordinate list sorted by (row, col): a non-unique compressed row level over a singleton column level."""
    rows = _i32(rows)
    return Tensor([("nonunique", n_rows, np.array([0, rows.shape[0]], dtype=np.int32), rows),
                   ("singleton", n_cols, cols)])


def _pack(ops):
    arr = (_Tensor * len(ops))()
    for t, o in enumerate(ops):
        arr[t] = o.c
    return arr


def total_cost(ops, tail_extent=0) -> int:
    return int(lib().ora_total_cost(_pack(ops), len(ops), C.c_int64(tail_extent)))


def find_partition(ops, Q, tail_extent=0):
    """Algorithm 1 for one query.  Returns (coord[dc], posn[k, d], cost)."""
    k, d = len(ops), ops[0].nlevels
    dc = d + (1 if tail_extent > 0 else 0)
    coord = np.zeros(dc, dtype=np.int64)
    posn = np.zeros((k, d), dtype=np.int64)
    cost = C.c_int64(0)
    rc = lib().ora_find_partition(_pack(ops), k, d, C.c_int64(tail_extent), C.c_int64(int(Q)),
                                  coord.ctypes.data_as(C.c_void_p), posn.ctypes.data_as(C.c_void_p),
                                  C.byref(cost))
    if rc:
        raise ValueError("ora_find_partition rejected its arguments")
    return coord, posn, int(cost.value)


def partition(ops, P, queries=None, tail_extent=0):
    """All P+1 boundaries.  Returns dict(coord[P+1, dc], posn[P+1, k, d], cost[P+1])."""
    k, d = len(ops), ops[0].nlevels
    dc = d + (1 if tail_extent > 0 else 0)
    coord = np.zeros((P + 1, dc), dtype=np.int64)
    posn = np.zeros((P + 1, k, d), dtype=np.int64)
    cost = np.zeros(P + 1, dtype=np.int64)
    qp = None
    if queries is not None:
        queries = np.ascontiguousarray(queries, dtype=np.int64)
        assert queries.shape[0] == P + 1
        qp = queries.ctypes.data_as(C.c_void_p)
    rc = lib().ora_partition(_pack(ops), k, d, C.c_int64(tail_extent), C.c_int64(P), qp,
                             coord.ctypes.data_as(C.c_void_p), posn.ctypes.data_as(C.c_void_p),
                             cost.ctypes.data_as(C.c_void_p))
    if rc:
        raise ValueError("ora_partition rejected its arguments")
    return {"coord": coord, "posn": posn, "cost": cost}


def partition_csr64(pos, row_crd, n_cols, P):
    """Algorithm 1 (Section 3.2) for ONE CSR operand whose positions do not fit 32 bits, in plain Python
    integers (the C oracle above describes operands with int32 arrays).  Cost functions of Section 4.2.2:
    C_i(x) = stored non-zeros in the rows before x = pos[x] (pos[0] = 0); C_j(c | x) = entries of row x in
    columns before c.  `pos`: integer array [n_rows + 1]; `row_crd(r)`: the sorted column coordinates
    of row r (only the rows that hold a boundary are asked for); queries Q_p = floor(p * Q_total / P).
    Conventions as partition(): boundary 0 is the origin, boundary P (and any query that reaches
    Q_total) the end; on a flat stretch of a cost function the highest coordinate is taken.
    Returns dict(coord[P+1, 2], posn[P+1, 2], cost[P+1]) of int64 (k = 1: posn has no operand axis)."""
    n_rows = len(pos) - 1
    base = int(pos[0])
    total = int(pos[n_rows]) - base
    coord = np.zeros((P + 1, 2), dtype=np.int64)
    posn = np.zeros((P + 1, 2), dtype=np.int64)
    cost = np.zeros(P + 1, dtype=np.int64)
    for p in range(P + 1):
        Q = (p * total) // P
        if p == 0:
            posn[p] = (0, base)
            continue
        if p == P or Q >= total:
            coord[p] = (n_rows, 0)
            posn[p] = (n_rows, int(pos[n_rows]))
            cost[p] = total
            continue
        # level 0: the highest row x in [0, n_rows] whose cost C_i(x) does not exceed the query
        lo, hi = 0, n_rows
        while lo < hi:
            x = lo + (hi - lo + 1) // 2
            if int(pos[x]) - base <= Q:
                lo = x
            else:
                hi = x - 1
        x0 = lo
        R = Q - (int(pos[x0]) - base)
        # level 1: the highest column c in [0, n_cols] with C_j(c | x0) <= the residual
        crd = np.asarray(row_crd(x0))
        before = lambda c: int(np.searchsorted(crd, c, side="left"))      # entries of the row in columns < c
        lo, hi = 0, n_cols
        while lo < hi:
            c = lo + (hi - lo + 1) // 2
            if before(c) <= R:
                lo = c
            else:
                hi = c - 1
        x1 = lo
        R -= before(x1)
        coord[p] = (x0, x1)
        posn[p] = (x0, int(pos[x0]) + before(x1))
        cost[p] = Q - R
    return {"coord": coord, "posn": posn, "cost": cost}


def partition_rowcost(ops, P, row_cost, queries=None):
    """All P+1 boundaries of two-level operands under the row-aware cost (every level-0 position costs
    `row_cost` on top of its stored non-zeros).  Same result layout as partition()."""
    k = len(ops)
    assert ops[0].nlevels == 2
    coord = np.zeros((P + 1, 2), dtype=np.int64)
    posn = np.zeros((P + 1, k, 2), dtype=np.int64)
    cost = np.zeros(P + 1, dtype=np.int64)
    qp = None
    if queries is not None:
        queries = np.ascontiguousarray(queries, dtype=np.int64)
        assert queries.shape[0] == P + 1
        qp = queries.ctypes.data_as(C.c_void_p)
    rc = lib().ora_partition_rowcost(_pack(ops), k, C.c_int64(row_cost), C.c_int64(P), qp,
                                     coord.ctypes.data_as(C.c_void_p), posn.ctypes.data_as(C.c_void_p),
                                     cost.ctypes.data_as(C.c_void_p))
    if rc:
        raise ValueError("ora_partition_rowcost rejected its arguments")
    return {"coord": coord, "posn": posn, "cost": cost}


def spmv(pos, crd, val, x):
    """Returns (y, s) as float64: y = A x, s_i = sum_j |A_ij x_j|."""
    pos, crd = _i32(pos), _i32(crd)
    n = pos.shape[0] - 1
    y = np.empty(n, dtype=np.float64)
    s = np.empty(n, dtype=np.float64)
    if val.dtype == np.float64:
        val, x = np.ascontiguousarray(val), np.ascontiguousarray(x, dtype=np.float64)
        fn = lib().ora_spmv_f64
    else:
        val, x = np.ascontiguousarray(val, dtype=np.float32), np.ascontiguousarray(x, dtype=np.float32)
        fn = lib().ora_spmv_f32
    fn(C.c_int64(n), pos.ctypes.data_as(C.c_void_p), crd.ctypes.data_as(C.c_void_p),
       val.ctypes.data_as(C.c_void_p), x.ctypes.data_as(C.c_void_p),
       y.ctypes.data_as(C.c_void_p), s.ctypes.data_as(C.c_void_p))
    return y, s


def spmm(pos, crd, val, B):
    """Returns (C, S) as float64 [n_rows, n]."""
    pos, crd = _i32(pos), _i32(crd)
    n_rows = pos.shape[0] - 1
    B = np.ascontiguousarray(B)
    n = B.shape[1]
    out = np.empty((n_rows, n), dtype=np.float64)
    sab = np.empty((n_rows, n), dtype=np.float64)
    if val.dtype == np.float64:
        val, B = np.ascontiguousarray(val), B.astype(np.float64, copy=False)
        fn = lib().ora_spmm_f64
    else:
        val, B = np.ascontiguousarray(val, dtype=np.float32), B.astype(np.float32, copy=False)
        fn = lib().ora_spmm_f32
    fn(C.c_int64(n_rows), pos.ctypes.data_as(C.c_void_p), crd.ctypes.data_as(C.c_void_p),
       val.ctypes.data_as(C.c_void_p), B.ctypes.data_as(C.c_void_p), C.c_int64(n), C.c_int64(n),
       out.ctypes.data_as(C.c_void_p), sab.ctypes.data_as(C.c_void_p))
    return out, sab


def _ptr_array(arrs):
    a = (C.c_void_p * len(arrs))()
    for t, x in enumerate(arrs):
        a[t] = x.ctypes.data
    return a


def _vals(vals):
    is64 = vals[0].dtype == np.float64
    dt = np.float64 if is64 else np.float32
    return [np.ascontiguousarray(v, dtype=dt) for v in vals], int(is64)


def spadd_vec(idxs, vals):
    """Union add of k sparse vectors.  Returns (idx int32, val f64, abs f64)."""
    k = len(idxs)
    idxs = [_i32(i) for i in idxs]
    vals, is64 = _vals(vals)
    nnz = np.array([i.shape[0] for i in idxs], dtype=np.int64)
    cap = int(nnz.sum())
    oi = np.empty(cap, dtype=np.int32)
    ov = np.empty(cap, dtype=np.float64)
    oa = np.empty(cap, dtype=np.float64)
    n = lib().ora_spadd_vec(k, _ptr_array(idxs), _ptr_array(vals), nnz.ctypes.data_as(C.c_void_p),
                            is64, oi.ctypes.data_as(C.c_void_p), ov.ctypes.data_as(C.c_void_p),
                            oa.ctypes.data_as(C.c_void_p))
    if n < 0:
        raise ValueError("ora_spadd_vec rejected its arguments")
    return oi[:n].copy(), ov[:n].copy(), oa[:n].copy()


def spadd_dcsr(mats):
    """Union add of k DCSR matrices given as dicts(pos0, crd0, pos1, crd1, val).
    Returns dict(pos0, crd0, pos1, crd1 int32; val, abs float64)."""
    k = len(mats)
    p0 = [_i32(m["pos0"]) for m in mats]
    c0 = [_i32(m["crd0"]) for m in mats]
    p1 = [_i32(m["pos1"]) for m in mats]
    c1 = [_i32(m["crd1"]) for m in mats]
    vals, is64 = _vals([m["val"] for m in mats])
    cap_r = sum(c.shape[0] for c in c0)
    cap_n = sum(c.shape[0] for c in c1)
    o_p0 = np.zeros(2, dtype=np.int32)
    o_c0 = np.empty(cap_r, dtype=np.int32)
    o_p1 = np.empty(cap_r + 1, dtype=np.int32)
    o_c1 = np.empty(cap_n, dtype=np.int32)
    o_v = np.empty(cap_n, dtype=np.float64)
    o_a = np.empty(cap_n, dtype=np.float64)
    counts = np.zeros(2, dtype=np.int64)
    rc = lib().ora_spadd_dcsr(k, _ptr_array(p0), _ptr_array(c0), _ptr_array(p1), _ptr_array(c1),
                              _ptr_array(vals), is64,
                              o_p0.ctypes.data_as(C.c_void_p), o_c0.ctypes.data_as(C.c_void_p),
                              o_p1.ctypes.data_as(C.c_void_p), o_c1.ctypes.data_as(C.c_void_p),
                              o_v.ctypes.data_as(C.c_void_p), o_a.ctypes.data_as(C.c_void_p),
                              counts.ctypes.data_as(C.c_void_p))
    if rc:
        raise ValueError("ora_spadd_dcsr rejected its arguments")
    nr, nz = int(counts[0]), int(counts[1])
    return {"pos0": o_p0, "crd0": o_c0[:nr].copy(), "pos1": o_p1[:nr + 1].copy(),
            "crd1": o_c1[:nz].copy(), "val": o_v[:nz].copy(), "abs": o_a[:nz].copy()}


def spadd_csf3(tens):
    """Union add of k third-order CSF tensors given as dicts(pos0, crd0, pos1, crd1, pos2, crd2, val).
    Returns dict(pos0, crd0, pos1, crd1, pos2, crd2 int32; val, abs float64)."""
    k = len(tens)
    arr = {n: [_i32(t[n]) for t in tens] for n in ("pos0", "crd0", "pos1", "crd1", "pos2", "crd2")}
    vals, is64 = _vals([t["val"] for t in tens])
    cap = [sum(c.shape[0] for c in arr[n]) for n in ("crd0", "crd1", "crd2")]
    o_p0 = np.zeros(2, dtype=np.int32)
    o_c0 = np.empty(cap[0], dtype=np.int32)
    o_p1 = np.empty(cap[0] + 1, dtype=np.int32)
    o_c1 = np.empty(cap[1], dtype=np.int32)
    o_p2 = np.empty(cap[1] + 1, dtype=np.int32)
    o_c2 = np.empty(cap[2], dtype=np.int32)
    o_v = np.empty(cap[2], dtype=np.float64)
    o_a = np.empty(cap[2], dtype=np.float64)
    counts = np.zeros(3, dtype=np.int64)
    p = lambda a: a.ctypes.data_as(C.c_void_p)
    rc = lib().ora_spadd_csf3(k, _ptr_array(arr["pos0"]), _ptr_array(arr["crd0"]), _ptr_array(arr["pos1"]),
                              _ptr_array(arr["crd1"]), _ptr_array(arr["pos2"]), _ptr_array(arr["crd2"]),
                              _ptr_array(vals), is64, p(o_p0), p(o_c0), p(o_p1), p(o_c1), p(o_p2), p(o_c2),
                              p(o_v), p(o_a), p(counts))
    if rc:
        raise ValueError("ora_spadd_csf3 rejected its arguments")
    n0, n1, n2 = (int(v) for v in counts)
    return {"pos0": o_p0, "crd0": o_c0[:n0].copy(), "pos1": o_p1[:n0 + 1].copy(), "crd1": o_c1[:n1].copy(),
            "pos2": o_p2[:n1 + 1].copy(), "crd2": o_c2[:n2].copy(), "val": o_v[:n2].copy(), "abs": o_a[:n2].copy()}


def spadd_csr(mats):
    """Union add of k CSR matrices given as dicts(pos, crd, val).
    Returns dict(pos, crd int32; val, abs float64)."""
    k = len(mats)
    pos = [_i32(m["pos"]) for m in mats]
    crd = [_i32(m["crd"]) for m in mats]
    vals, is64 = _vals([m["val"] for m in mats])
    n_rows = pos[0].shape[0] - 1
    cap = sum(c.shape[0] for c in crd)
    o_pos = np.empty(n_rows + 1, dtype=np.int32)
    o_crd = np.empty(cap, dtype=np.int32)
    o_v = np.empty(cap, dtype=np.float64)
    o_a = np.empty(cap, dtype=np.float64)
    nz = lib().ora_spadd_csr(k, C.c_int64(n_rows), _ptr_array(pos), _ptr_array(crd), _ptr_array(vals),
                             is64, o_pos.ctypes.data_as(C.c_void_p), o_crd.ctypes.data_as(C.c_void_p),
                             o_v.ctypes.data_as(C.c_void_p), o_a.ctypes.data_as(C.c_void_p))
    if nz < 0:
        raise ValueError("ora_spadd_csr rejected its arguments")
    return {"pos": o_pos, "crd": o_crd[:nz].copy(), "val": o_v[:nz].copy(), "abs": o_a[:nz].copy()}


def spmul_vec(idxs, vals):
    """Intersection multiply of k sparse vectors.  Returns (idx int32, val f64, abs f64)."""
    k = len(idxs)
    idxs = [_i32(i) for i in idxs]
    vals, is64 = _vals(vals)
    nnz = np.array([i.shape[0] for i in idxs], dtype=np.int64)
    cap = int(nnz.min()) if k else 0
    oi = np.empty(cap, dtype=np.int32)
    ov = np.empty(cap, dtype=np.float64)
    oa = np.empty(cap, dtype=np.float64)
    n = lib().ora_spmul_vec(k, _ptr_array(idxs), _ptr_array(vals), nnz.ctypes.data_as(C.c_void_p),
                            is64, oi.ctypes.data_as(C.c_void_p), ov.ctypes.data_as(C.c_void_p),
                            oa.ctypes.data_as(C.c_void_p))
    if n < 0:
        raise ValueError("ora_spmul_vec rejected its arguments")
    return oi[:n].copy(), ov[:n].copy(), oa[:n].copy()


def spmul_csr(mats):
    """Hadamard product of k CSR matrices given as dicts(pos, crd, val).
    Returns dict(pos, crd int32; val, abs float64)."""
    k = len(mats)
    pos = [_i32(m["pos"]) for m in mats]
    crd = [_i32(m["crd"]) for m in mats]
    vals, is64 = _vals([m["val"] for m in mats])
    n_rows = pos[0].shape[0] - 1
    cap = min(c.shape[0] for c in crd)
    o_pos = np.empty(n_rows + 1, dtype=np.int32)
    o_crd = np.empty(cap, dtype=np.int32)
    o_v = np.empty(cap, dtype=np.float64)
    o_a = np.empty(cap, dtype=np.float64)
    nz = lib().ora_spmul_csr(k, C.c_int64(n_rows), _ptr_array(pos), _ptr_array(crd), _ptr_array(vals),
                             is64, o_pos.ctypes.data_as(C.c_void_p), o_crd.ctypes.data_as(C.c_void_p),
                             o_v.ctypes.data_as(C.c_void_p), o_a.ctypes.data_as(C.c_void_p))
    if nz < 0:
        raise ValueError("ora_spmul_csr rejected its arguments")
    return {"pos": o_pos, "crd": o_crd[:nz].copy(), "val": o_v[:nz].copy(), "abs": o_a[:nz].copy()}


def spmul_dcsr(mats):
    """Hadamard product of k DCSR matrices given as dicts(pos0, crd0, pos1, crd1, val).
    Returns dict(pos0, crd0, pos1, crd1 int32; val, abs float64)."""
    k = len(mats)
    p0 = [_i32(m["pos0"]) for m in mats]
    c0 = [_i32(m["crd0"]) for m in mats]
    p1 = [_i32(m["pos1"]) for m in mats]
    c1 = [_i32(m["crd1"]) for m in mats]
    vals, is64 = _vals([m["val"] for m in mats])
    cap_r = min(c.shape[0] for c in c0)
    cap_n = min(c.shape[0] for c in c1)
    o_p0 = np.zeros(2, dtype=np.int32)
    o_c0 = np.empty(cap_r, dtype=np.int32)
    o_p1 = np.empty(cap_r + 1, dtype=np.int32)
    o_c1 = np.empty(cap_n, dtype=np.int32)
    o_v = np.empty(cap_n, dtype=np.float64)
    o_a = np.empty(cap_n, dtype=np.float64)
    counts = np.zeros(2, dtype=np.int64)
    rc = lib().ora_spmul_dcsr(k, _ptr_array(p0), _ptr_array(c0), _ptr_array(p1), _ptr_array(c1),
                              _ptr_array(vals), is64,
                              o_p0.ctypes.data_as(C.c_void_p), o_c0.ctypes.data_as(C.c_void_p),
                              o_p1.ctypes.data_as(C.c_void_p), o_c1.ctypes.data_as(C.c_void_p),
                              o_v.ctypes.data_as(C.c_void_p), o_a.ctypes.data_as(C.c_void_p),
                              counts.ctypes.data_as(C.c_void_p))
    if rc:
        raise ValueError("ora_spmul_dcsr rejected its arguments")
    nr, nz = int(counts[0]), int(counts[1])
    return {"pos0": o_p0, "crd0": o_c0[:nr].copy(), "pos1": o_p1[:nr + 1].copy(),
            "crd1": o_c1[:nz].copy(), "val": o_v[:nz].copy(), "abs": o_a[:nz].copy()}


def recursive_partition_dcsr(mats, n_cols, P, queries=None):
    """Algorithm 2 for the Hadamard product of k DCSR matrices (dicts as above; val unused).
    Returns dict(rows[M], rpos[k, M], T[M], Tprime[M+1], coord[P+1, 2] = (i', j),
    lpos[P+1, k], before[P+1, k], cost[P+1])."""
    k = len(mats)
    p0 = [_i32(m["pos0"]) for m in mats]
    c0 = [_i32(m["crd0"]) for m in mats]
    p1 = [_i32(m["pos1"]) for m in mats]
    c1 = [_i32(m["crd1"]) for m in mats]
    cap = max(1, min(c.shape[0] for c in c0))
    rows = np.zeros(cap, dtype=np.int64)
    rpos = np.zeros((k, cap), dtype=np.int64)
    T = np.zeros(cap, dtype=np.int64)
    lib().ora_remap_rows.restype = C.c_int64
    M = int(lib().ora_remap_rows(k, _ptr_array(p0), _ptr_array(c0), _ptr_array(p1), C.c_int64(cap),
                                 rows.ctypes.data_as(C.c_void_p), rpos.ctypes.data_as(C.c_void_p),
                                 T.ctypes.data_as(C.c_void_p)))
    if M < 0:
        raise ValueError("ora_remap_rows rejected its arguments")
    Tprime = np.zeros(M + 1, dtype=np.int64)
    coord = np.zeros((P + 1, 2), dtype=np.int64)
    lpos = np.zeros((P + 1, k), dtype=np.int64)
    before = np.zeros((P + 1, k), dtype=np.int64)
    cost = np.zeros(P + 1, dtype=np.int64)
    qp = None
    if queries is not None:
        queries = np.ascontiguousarray(queries, dtype=np.int64)
        assert queries.shape[0] == P + 1
        qp = queries.ctypes.data_as(C.c_void_p)
    rc = lib().ora_recursive_partition_dcsr(k, _ptr_array(p1), _ptr_array(c1), C.c_int64(n_cols),
                                            C.c_int64(M), C.c_int64(cap),
                                            rpos.ctypes.data_as(C.c_void_p), T.ctypes.data_as(C.c_void_p),
                                            C.c_int64(P), qp, Tprime.ctypes.data_as(C.c_void_p),
                                            coord.ctypes.data_as(C.c_void_p), lpos.ctypes.data_as(C.c_void_p),
                                            before.ctypes.data_as(C.c_void_p), cost.ctypes.data_as(C.c_void_p))
    if rc:
        raise ValueError("ora_recursive_partition_dcsr rejected its arguments")
    return {"rows": rows[:M].copy(), "rpos": rpos[:, :M].copy(), "T": T[:M].copy(), "Tprime": Tprime,
            "coord": coord, "lpos": lpos, "before": before, "cost": cost}


def _coo_combine(fn, mats, cap):
    k = len(mats)
    rows = [_i32(m["row"]) for m in mats]
    cols = [_i32(m["col"]) for m in mats]
    vals, is64 = _vals([m["val"] for m in mats])
    nnz = np.array([r.shape[0] for r in rows], dtype=np.int64)
    o_r = np.empty(cap, dtype=np.int32)
    o_c = np.empty(cap, dtype=np.int32)
    o_v = np.empty(cap, dtype=np.float64)
    o_a = np.empty(cap, dtype=np.float64)
    n = fn(k, _ptr_array(rows), _ptr_array(cols), _ptr_array(vals), nnz.ctypes.data_as(C.c_void_p), is64,
           o_r.ctypes.data_as(C.c_void_p), o_c.ctypes.data_as(C.c_void_p), o_v.ctypes.data_as(C.c_void_p),
           o_a.ctypes.data_as(C.c_void_p))
    if n < 0:
        raise ValueError("the COO oracle rejected its arguments")
    return {"row": o_r[:n].copy(), "col": o_c[:n].copy(), "val": o_v[:n].copy(), "abs": o_a[:n].copy()}


def spadd_coo(mats):
    """Union add of k COO matrices given as dicts(row, col, val) sorted by (row, col)."""
    return _coo_combine(lib().ora_spadd_coo, mats, max(1, sum(len(m["row"]) for m in mats)))


def spmul_coo(mats):
    """Hadamard product of k COO matrices given as dicts(row, col, val) sorted by (row, col)."""
    return _coo_combine(lib().ora_spmul_coo, mats, max(1, min(len(m["row"]) for m in mats)))
