"""The C-ABI library loads and exports every symbol include/nacho.h declares
(no compute calls: this runs without a GPU)."""
import ctypes
import os
import re

import pytest

from paper_2604_17198_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "nacho.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nacho_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    if not os.path.exists(build.LIB):
        pytest.fail(f"{build.LIB} not built; run `python -m paper_2604_17198_amd.build`")
    lib = ctypes.CDLL(build.LIB)
    names = _declared()
    assert {"nacho_partition", "nacho_spmv", "nacho_spadd_k", "nacho_spmm"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"libnacho.so does not export {n}"
    assert sorted(binding.EXPORTS) == names


def test_host_side_helpers_run_without_a_gpu():
    lib = binding.lib()
    assert lib.nacho_version() >= 100
    assert binding.status_string(0) == "ok" and "workspace" in binding.status_string(-3)
    # automatic partition count: enough partitions that each fits a wavefront's staging buffer
    def csr_desc(nnz):
        t = binding._Tensor()
        t.nlevels = 2
        t.lvl[0].kind, t.lvl[0].extent = binding.DENSE, 1000
        t.lvl[1].kind, t.lvl[1].extent, t.lvl[1].count = binding.COMPRESSED, 1000, nnz
        return (binding._Tensor * 1)(t)

    def nparts(nnz, P=0):
        return lib.nacho_num_partitions(binding.OP_SPMV, ctypes.cast(csr_desc(nnz), ctypes.c_void_p), 1,
                                        binding.F64, 0, P)

    assert nparts(50_000_000) >= 50_000_000 // 4096 and nparts(0) == 1 and nparts(1000, 77) == 77


def test_argument_errors_are_reported_before_any_launch():
    lib = binding.lib()
    n = ctypes.c_size_t(0)
    assert lib.nacho_workspace_bytes(binding.OP_SPMV, None, 1, binding.F64, 0, 0, ctypes.byref(n)) == -1
    t = binding._Tensor()
    t.nlevels = 2
    t.lvl[0].kind, t.lvl[0].extent = binding.DENSE, 10
    t.lvl[1].kind, t.lvl[1].extent, t.lvl[1].count = binding.COMPRESSED, 10, 5
    arr = (binding._Tensor * 1)(t)
    assert lib.nacho_workspace_bytes(binding.OP_SPMV, ctypes.cast(arr, ctypes.c_void_p), 1,
                                     binding.F64, 0, 0, ctypes.byref(n)) == 0 and n.value > 0
    # null x / y, bad dtype
    assert lib.nacho_spmv(ctypes.cast(arr, ctypes.c_void_p), None, None, binding.F64, 0, None, 0, None) == -1
    # 3 levels are not supported
    t.nlevels = 3
    arr = (binding._Tensor * 1)(t)
    assert lib.nacho_workspace_bytes(binding.OP_SPMV, ctypes.cast(arr, ctypes.c_void_p), 1,
                                     binding.F64, 0, 0, ctypes.byref(n)) == -2
