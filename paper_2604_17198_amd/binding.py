"""Thin ctypes binding over libnacho.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU, passes their
device pointers through the C ABI declared in include/nacho.h and returns the
status code handling to `_check`.  PyTorch is used for device memory and the
current stream; no step of the hot path runs in Python or in torch.

The library must have been built (`paper_2604_17198_amd.build.build()`); a
missing library is an error, there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

from . import build as _build

F32, F64 = 0, 1
DENSE, COMPRESSED, NONUNIQUE, SINGLETON = 0, 1, 2, 3
OP_PARTITION, OP_SPMV, OP_SPMM, OP_SPADD, OP_SPMUL = 0, 1, 2, 3, 4
MAX_OPERANDS, MAX_LEVELS = 8, 3

EXPORTS = [
    "nacho_version", "nacho_status_string", "nacho_num_partitions", "nacho_workspace_bytes",
    "nacho_partition", "nacho_spmv", "nacho_spmm", "nacho_spadd_k", "nacho_spmul_k", "nacho_workspace_parts",
    "nacho_validate", "nacho_profile_enable", "nacho_profile_read", "nacho_spmv_static",
    "nacho_static_scratch_bytes", "nacho_instrument", "nacho_instrument_record_bytes",
    "nacho_probe", "nacho_merge_wavefronts", "nacho_rowcost_partitions", "nacho_partition_rowcost",
    "nacho_spmv_rowcost", "nacho_partition_csr64", "nacho_spmv_fused", "nacho_spadd_fused",
]


class NachoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class _Level(C.Structure):
    _fields_ = [("kind", C.c_int32), ("extent", C.c_int64), ("pos", C.c_void_p),
                ("crd", C.c_void_p), ("count", C.c_int64)]


class _Tensor(C.Structure):
    _fields_ = [("nlevels", C.c_int32), ("lvl", _Level * MAX_LEVELS), ("val", C.c_void_p)]


class _Parts(C.Structure):
    _fields_ = [("k", C.c_int32), ("d", C.c_int32), ("P", C.c_int64), ("coord", C.c_void_p),
                ("posn", C.c_void_p), ("cost", C.c_void_p)]


class _SparseOut(C.Structure):
    _fields_ = [("pos0", C.c_void_p), ("crd0", C.c_void_p), ("pos1", C.c_void_p),
                ("crd1", C.c_void_p), ("val", C.c_void_p), ("cap_rows", C.c_int64),
                ("cap_nnz", C.c_int64), ("counts", C.c_void_p), ("status", C.c_void_p),
                ("pos2", C.c_void_p), ("crd2", C.c_void_p), ("cap_fibres", C.c_int64)]


_lib = None
_libs = {}
_instrumented = False


def select_library(instrumented: bool):
    """Route all calls to libnacho.so (default) or to libnacho_instr.so, the instrumented build."""
    global _lib, _instrumented
    _instrumented = bool(instrumented)
    _lib = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None and _instrumented in _libs:
        _lib = _libs[_instrumented]
    if _lib is None:
        path = _build.LIB_INSTR if _instrumented else _build.LIB
        if not os.path.exists(path):
            raise RuntimeError(
                f"{path} is missing: build it with `python -m paper_2604_17198_amd.build` "
                "(the HIP path has no fallback)")
        L = C.CDLL(path)
        L.nacho_status_string.restype = C.c_char_p
        L.nacho_num_partitions.restype = C.c_int64
        L.nacho_num_partitions.argtypes = [C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_int64, C.c_int64]
        L.nacho_workspace_bytes.argtypes = [C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_int64,
                                            C.c_int64, C.POINTER(C.c_size_t)]
        L.nacho_partition.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_int64, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.nacho_spmv.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64,
                                 C.c_void_p, C.c_size_t, C.c_void_p]
        L.nacho_spmv_static.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_void_p]
        L.nacho_static_scratch_bytes.restype = C.c_size_t
        L.nacho_spmm.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_int64,
                                 C.c_int32, C.c_int64, C.c_void_p, C.c_size_t, C.c_void_p]
        L.nacho_spadd_k.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int64, C.c_void_p,
                                    C.c_void_p, C.c_size_t, C.c_void_p]
        L.nacho_spmul_k.argtypes = L.nacho_spadd_k.argtypes
        L.nacho_spadd_fused.argtypes = L.nacho_spadd_k.argtypes
        L.nacho_workspace_parts.argtypes = [C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_int64, C.c_int64,
                                            C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p]
        L.nacho_profile_read.argtypes = [C.c_void_p, C.c_void_p, C.c_int32]
        L.nacho_validate.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.nacho_instrument.argtypes = [C.c_void_p, C.c_int64]
        L.nacho_spmv_fused.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_size_t,
                                       C.c_void_p]
        L.nacho_partition_csr64.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int64,
                                            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.nacho_rowcost_partitions.restype = C.c_int64
        L.nacho_rowcost_partitions.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_int64]
        L.nacho_partition_rowcost.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p]
        L.nacho_spmv_rowcost.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int64,
                                         C.c_void_p, C.c_size_t, C.c_void_p]
        L.nacho_probe.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_int64, C.c_void_p]
        _libs[_instrumented] = L
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().nacho_status_string(C.c_int32(status)).decode()


def _check(status: int, where: str):
    if status != 0:
        raise NachoError(status, where)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def dtype_code(dt) -> int:
    if dt == torch.float32:
        return F32
    if dt == torch.float64:
        return F64
    raise TypeError(f"unsupported value type {dt}")


# --------------------------------------------------------------------------- #
# operand descriptors (host structs holding device pointers)
# --------------------------------------------------------------------------- #
class Operand:
    """Keeps the tensors alive and exposes the C descriptor."""

    def __init__(self, levels, val=None):
        self.keep = []
        c = _Tensor()
        c.nlevels = len(levels)
        for m, l in enumerate(levels):
            c.lvl[m].extent = int(l["extent"])
            if l["kind"] == "dense":
                c.lvl[m].kind = DENSE
                c.lvl[m].pos = None
                c.lvl[m].crd = None
                c.lvl[m].count = 0
            elif l["kind"] in ("nonunique", "singleton"):
                crd = l["crd"]
                assert crd.dtype == torch.int32
                self.keep.append(crd)
                c.lvl[m].kind = NONUNIQUE if l["kind"] == "nonunique" else SINGLETON
                c.lvl[m].pos = None
                c.lvl[m].crd = crd.data_ptr() if crd.numel() else None
                c.lvl[m].count = int(crd.numel())
            else:
                pos, crd = l["pos"], l["crd"]
                assert pos.dtype == torch.int32 and crd.dtype == torch.int32
                self.keep += [pos, crd]
                c.lvl[m].kind = COMPRESSED
                c.lvl[m].pos = pos.data_ptr()
                c.lvl[m].crd = crd.data_ptr() if crd.numel() else None
                c.lvl[m].count = int(crd.numel())
        if val is not None:
            self.keep.append(val)
            c.val = val.data_ptr() if val.numel() else None
        self.c = c
        self.nlevels = len(levels)
        self.nnz = int(levels[-1]["crd"].numel())
        self.val = val


def vector(idx, extent, val=None):
    pos = torch.tensor([0, idx.numel()], dtype=torch.int32, device=idx.device)
    return Operand([{"kind": "compressed", "extent": extent, "pos": pos, "crd": idx}], val)


def csr(pos, crd, n_rows, n_cols, val=None):
    return Operand([{"kind": "dense", "extent": n_rows},
                    {"kind": "compressed", "extent": n_cols, "pos": pos, "crd": crd}], val)


def dcsr(pos0, crd0, pos1, crd1, n_rows, n_cols, val=None):
    return Operand([{"kind": "compressed", "extent": n_rows, "pos": pos0, "crd": crd0},
                    {"kind": "compressed", "extent": n_cols, "pos": pos1, "crd": crd1}], val)


def csf3(pos0, crd0, pos1, crd1, pos2, crd2, shape, val=None):
    """Third-order tensor, three compressed levels (nacho_partition, nacho_spadd_k)."""
    return Operand([{"kind": "compressed", "extent": shape[0], "pos": pos0, "crd": crd0},
                    {"kind": "compressed", "extent": shape[1], "pos": pos1, "crd": crd1},
                    {"kind": "compressed", "extent": shape[2], "pos": pos2, "crd": crd2}], val)


def coo(rows, cols, n_rows, n_cols, val=None):
    """Coordinate list sorted by (row, column), no pair twice."""
    return Operand([{"kind": "nonunique", "extent": n_rows, "crd": rows},
                    {"kind": "singleton", "extent": n_cols, "crd": cols}], val)


def _pack(ops):
    arr = (_Tensor * len(ops))()
    for t, o in enumerate(ops):
        arr[t] = o.c
    return arr


# --------------------------------------------------------------------------- #
# entry points
# --------------------------------------------------------------------------- #
def version() -> int:
    return int(lib().nacho_version())


def num_partitions(op, ops, dtype, n_dense=0, P=0) -> int:
    arr = _pack(ops)
    return int(lib().nacho_num_partitions(op, C.cast(arr, C.c_void_p), len(ops), dtype, n_dense, P))


def workspace_bytes(op, ops, dtype, n_dense=0, P=0) -> int:
    n = C.c_size_t(0)
    arr = _pack(ops)
    _check(lib().nacho_workspace_bytes(op, C.cast(arr, C.c_void_p), len(ops), dtype, n_dense, P,
                                       C.byref(n)), "nacho_workspace_bytes")
    return int(n.value)


def _workspace(nbytes, device):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def nacho_partition(ops, P, queries=None, cost_scale=1):
    """Boundaries 0..P.  Returns dict(coord[P+1, d], posn[P+1, k, d] int32, cost[P+1] int64)
    as device tensors."""
    k, d = len(ops), ops[0].nlevels
    dev = ops[0].keep[0].device
    coord = torch.empty((P + 1, d), dtype=torch.int32, device=dev)
    posn = torch.empty((P + 1, k, d), dtype=torch.int32, device=dev)
    cost = torch.empty(P + 1, dtype=torch.int64, device=dev)
    parts = _Parts(k, d, P, coord.data_ptr(), posn.data_ptr(), cost.data_ptr())
    arr = _pack(ops)
    if queries is not None:
        assert queries.dtype == torch.int64 and queries.numel() == P + 1
    _check(lib().nacho_partition(C.cast(arr, C.c_void_p), k, cost_scale, P, _ptr(queries),
                                 C.byref(parts), None, 0, _stream()), "nacho_partition")
    return {"coord": coord, "posn": posn, "cost": cost}


def nacho_partition_csr64(pos, crd, n_rows, n_cols, P):
    """All P+1 boundaries of one CSR operand with 64-bit positions (pos: int64 device tensor).
    Returns dict(coord int32 [P+1, 2], posn int64 [P+1, 2], cost int64 [P+1]); enqueues only."""
    dev = pos.device
    assert pos.dtype == torch.int64 and (crd is None or crd.dtype == torch.int32)
    nnz = int((pos[-1] - pos[0]).item())
    coord = torch.empty((P + 1, 2), dtype=torch.int32, device=dev)
    posn = torch.empty((P + 1, 2), dtype=torch.int64, device=dev)
    cost = torch.empty(P + 1, dtype=torch.int64, device=dev)
    _check(lib().nacho_partition_csr64(_ptr(pos), _ptr(crd), n_rows, n_cols, nnz, P, _ptr(coord), _ptr(posn),
                                       _ptr(cost), _stream()), "nacho_partition_csr64")
    return {"coord": coord, "posn": posn, "cost": cost}


def workspace_parts(op, ops, dtype, ws, n_dense=0, P=0):
    """The partition table a fused call keeps in its workspace `ws` (valid after the call ran):
    dict(coord[P+1, d], posn[P+1, k, d] int32, cost[P+1] int64) as copies, plus 'P' and 'grain'."""
    parts = _Parts()
    grain = C.c_int64(0)
    arr = _pack(ops)
    _check(lib().nacho_workspace_parts(op, C.cast(arr, C.c_void_p), len(ops), dtype, n_dense, P, _ptr(ws),
                                       ws.numel(), C.byref(parts), C.byref(grain), _stream()),
           "nacho_workspace_parts")
    base = ws.data_ptr()
    k, d, Pe = parts.k, parts.d, int(parts.P)

    def view(ptr, count, dt, shape):
        off = ptr - base
        nbytes = count * (8 if dt == torch.int64 else 4)
        return ws[off:off + nbytes].view(dt).reshape(shape).clone()

    return {"coord": view(parts.coord, (Pe + 1) * d, torch.int32, (Pe + 1, d)),
            "posn": view(parts.posn, (Pe + 1) * k * d, torch.int32, (Pe + 1, k, d)),
            "cost": view(parts.cost, Pe + 1, torch.int64, (Pe + 1,)), "P": Pe, "grain": int(grain.value)}


def nacho_spmv(A: Operand, x, y=None, P=0, ws=None):
    """y = A x.  A is a CSR Operand with values; x, y device tensors of A's value type."""
    dt = dtype_code(x.dtype)
    if y is None:
        y = torch.empty(A.c.lvl[0].extent, dtype=x.dtype, device=x.device)
    if ws is None:
        ws = _workspace(workspace_bytes(OP_SPMV, [A], dt, 0, P), x.device)
    arr = _pack([A])
    _check(lib().nacho_spmv(C.cast(arr, C.c_void_p), _ptr(x), _ptr(y), dt, P, _ptr(ws),
                            ws.numel(), _stream()), "nacho_spmv")
    return y


def nacho_spmv_fused(A: Operand, x, y, ws=None):
    """y = A x without a partition pass: the executing wavefronts search their own boundaries."""
    dt = dtype_code(x.dtype)
    if ws is None:
        ws = _workspace(workspace_bytes(OP_SPMV, [A], dt, 0, 0), x.device)
    arr = _pack([A])
    _check(lib().nacho_spmv_fused(C.cast(arr, C.c_void_p), _ptr(x), _ptr(y), dt, _ptr(ws), ws.numel(), _stream()),
           "nacho_spmv_fused")
    return y


def nacho_spmv_static(A: Operand, x, y, P=0):
    """y = A x on the library's built-in scratch memory: no workspace, nothing allocated (y is the
    caller's)."""
    arr = _pack([A])
    _check(lib().nacho_spmv_static(C.cast(arr, C.c_void_p), _ptr(x), _ptr(y), dtype_code(x.dtype), P,
                                   _stream()), "nacho_spmv_static")
    return y


def static_scratch_bytes() -> int:
    return int(lib().nacho_static_scratch_bytes())


def rowcost_partitions(A: Operand, dtype, row_cost, P=0) -> int:
    arr = _pack([A])
    return int(lib().nacho_rowcost_partitions(C.cast(arr, C.c_void_p), dtype, row_cost, P))


def nacho_partition_rowcost(A: Operand, P, row_cost):
    """Boundaries 0..P of one CSR operand under the row-aware cost; result as nacho_partition."""
    dev = A.keep[0].device
    coord = torch.empty((P + 1, 2), dtype=torch.int32, device=dev)
    posn = torch.empty((P + 1, 1, 2), dtype=torch.int32, device=dev)
    cost = torch.empty(P + 1, dtype=torch.int64, device=dev)
    parts = _Parts(1, 2, P, coord.data_ptr(), posn.data_ptr(), cost.data_ptr())
    arr = _pack([A])
    _check(lib().nacho_partition_rowcost(C.cast(arr, C.c_void_p), row_cost, P, C.byref(parts), _stream()),
           "nacho_partition_rowcost")
    return {"coord": coord, "posn": posn, "cost": cost}


def nacho_spmv_rowcost(A: Operand, x, y, row_cost, P=0, ws=None):
    """y = A x on partitions balanced by non-zeros + row_cost per row."""
    dt = dtype_code(x.dtype)
    Pe = rowcost_partitions(A, dt, row_cost, P)
    if ws is None:
        ws = _workspace(workspace_bytes(OP_SPMV, [A], dt, 0, Pe), x.device)
    arr = _pack([A])
    _check(lib().nacho_spmv_rowcost(C.cast(arr, C.c_void_p), _ptr(x), _ptr(y), dt, row_cost, P, _ptr(ws),
                                    ws.numel(), _stream()), "nacho_spmv_rowcost")
    return y


def nacho_spmm(A: Operand, B, Cout=None, P=0, ws=None):
    """C = A B with B, C dense row-major device tensors."""
    dt = dtype_code(B.dtype)
    n = int(B.shape[1])
    if Cout is None:
        Cout = torch.empty((A.c.lvl[0].extent, n), dtype=B.dtype, device=B.device)
    if ws is None:
        ws = _workspace(workspace_bytes(OP_SPMM, [A], dt, n, P), B.device)
    arr = _pack([A])
    _check(lib().nacho_spmm(C.cast(arr, C.c_void_p), _ptr(B), n, int(B.stride(0)), _ptr(Cout),
                            int(Cout.stride(0)), dt, P, _ptr(ws), ws.numel(), _stream()), "nacho_spmm")
    return Cout


class SparseOut:
    """Caller-allocated result arrays of nacho_spadd_k."""

    def __init__(self, fmt, cap_rows, cap_nnz, dtype, device, n_rows=0, cap_fibres=0):
        """fmt "csf3": cap_rows is the capacity in slices, cap_fibres in fibres."""
        i32 = dict(dtype=torch.int32, device=device)
        self.fmt = fmt
        self.pos0 = torch.zeros(2, **i32) if fmt in ("dcsr", "csf3") else None
        self.crd0 = None
        if fmt in ("dcsr", "csf3"):
            self.crd0 = torch.empty(max(cap_rows, 1), **i32)
        elif fmt == "coo":
            self.crd0 = torch.empty(max(cap_nnz, 1), **i32)      # the rows of the result's entries
        n_pos1 = {"vector": 2, "coo": 2, "csr": n_rows + 1, "dcsr": cap_rows + 1, "csf3": cap_rows + 1}[fmt]
        self.pos1 = torch.zeros(n_pos1, **i32)
        self.crd1 = torch.empty(max(cap_fibres if fmt == "csf3" else cap_nnz, 1), **i32)
        self.pos2 = torch.zeros(cap_fibres + 1, **i32) if fmt == "csf3" else None
        self.crd2 = torch.empty(max(cap_nnz, 1), **i32) if fmt == "csf3" else None
        self.val = torch.empty(max(cap_nnz, 1), dtype=dtype, device=device)
        self.counts = torch.zeros(3, dtype=torch.int64, device=device)
        self.status = torch.zeros(1, dtype=torch.int32, device=device)
        self.c = _SparseOut(_ptr(self.pos0), _ptr(self.crd0), _ptr(self.pos1), _ptr(self.crd1),
                            _ptr(self.val), cap_rows, cap_nnz, _ptr(self.counts), _ptr(self.status),
                            _ptr(self.pos2), _ptr(self.crd2), cap_fibres)


def nacho_spadd_k(ops, out: SparseOut, P=0, ws=None):
    """Z = sum of the operands (union add).  Enqueues only; read out.counts / out.status after
    synchronising."""
    dt = dtype_code(ops[0].val.dtype)
    dev = ops[0].val.device
    if ws is None:
        ws = _workspace(workspace_bytes(OP_SPADD, ops, dt, 0, P), dev)
    arr = _pack(ops)
    _check(lib().nacho_spadd_k(C.cast(arr, C.c_void_p), len(ops), dt, P, C.byref(out.c), _ptr(ws),
                               ws.numel(), _stream()), "nacho_spadd_k")
    return out


def nacho_spadd_fused(ops, out: SparseOut, P=0, ws=None):
    """nacho_spadd_k on sparse vectors without a partition pass: the workgroups of the merge kernel search
    their own boundaries.  Enqueues only."""
    dt = dtype_code(ops[0].val.dtype)
    dev = ops[0].val.device
    if ws is None:
        ws = _workspace(workspace_bytes(OP_SPADD, ops, dt, 0, P), dev)
    arr = _pack(ops)
    _check(lib().nacho_spadd_fused(C.cast(arr, C.c_void_p), len(ops), dt, P, C.byref(out.c), _ptr(ws),
                                   ws.numel(), _stream()), "nacho_spadd_fused")
    return out


def nacho_spmul_k(ops, out: SparseOut, P=0, ws=None):
    """Z = product of the operands over the intersection of their coordinates (vectors, CSR, DCSR, COO).
    Enqueues only."""
    dt = dtype_code(ops[0].val.dtype)
    dev = ops[0].val.device
    if ws is None:
        ws = _workspace(workspace_bytes(OP_SPMUL, ops, dt, 0, P), dev)
    arr = _pack(ops)
    _check(lib().nacho_spmul_k(C.cast(arr, C.c_void_p), len(ops), dt, P, C.byref(out.c), _ptr(ws),
                               ws.numel(), _stream()), "nacho_spmul_k")
    return out


def nacho_validate(ops):
    """Checks the operands' preconditions on the device.  Returns (status, (operand, level, position))
    after synchronising: status 0, or -1 with the place of one violation."""
    dev = ops[0].keep[0].device
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    info = torch.zeros(3, dtype=torch.int64, device=dev)
    arr = _pack(ops)
    _check(lib().nacho_validate(C.cast(arr, C.c_void_p), len(ops), _ptr(status), _ptr(info), _stream()),
           "nacho_validate")
    torch.cuda.synchronize()
    return int(status.cpu()[0]), tuple(int(v) for v in info.cpu())


WAVE_RECORD = [("t_begin", "<u8"), ("t_end", "<u8"), ("cycles", "<u8"), ("items", "<u4"), ("rows", "<u4"),
               ("hw_id", "<u4"), ("xcc_id", "<u4")]


def instrument(records, capacity=None):
    """Instrumented library only: executing kernels log one WAVE_RECORD per wavefront into the
    device uint8 tensor `records` (None: stop logging)."""
    rb = int(lib().nacho_instrument_record_bytes())
    if records is None:
        _check(lib().nacho_instrument(None, 0), "nacho_instrument")
        return
    cap = records.numel() // rb if capacity is None else capacity
    _check(lib().nacho_instrument(_ptr(records), cap), "nacho_instrument")


def merge_wavefronts() -> int:
    return int(lib().nacho_merge_wavefronts())


PROBE_READ, PROBE_COPY, PROBE_GATHER = 0, 1, 2


def probe(kind, dst, src, nbytes, gathers=0):
    """Enqueue one of the library's kernels of known traffic (see nacho_probe)."""
    _check(lib().nacho_probe(kind, _ptr(dst), _ptr(src), nbytes, gathers, _stream()), "nacho_probe")


def profile_enable(on: bool):
    lib().nacho_profile_enable(1 if on else 0)


def profile_read():
    """[(kernel name, ms)] of the last fused call (synchronises)."""
    ms = (C.c_float * 16)()
    names = (C.c_char_p * 16)()
    n = lib().nacho_profile_read(C.cast(ms, C.c_void_p), C.cast(names, C.c_void_p), 16)
    if n < 0:
        raise NachoError(n, "nacho_profile_read")
    return [(names[i].decode(), float(ms[i])) for i in range(min(n, 16))]
