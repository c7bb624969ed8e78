"""GPU: nacho_spmv_static (the entry point that allocates nothing) against nacho_spmv, through the
C ABI, on two calls in a row, the second on a smaller matrix.  Both run the same kernels on the
same partitions, so the results must agree bit for bit (which is inside the 1e-12 / 1e-5 bar)."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2604_17198_amd import binding as nb
from paper_2604_17198_amd import workloads
from gpu_util import csr_operand, dev

pytestmark = pytest.mark.gpu


def _both(A, x, P):
    op, xd = csr_operand(A), dev(x)
    y_ref = torch.full((A["n_rows"],), float("nan"), dtype=xd.dtype, device="cuda")
    y_new = torch.full_like(y_ref, float("nan"))
    nb.nacho_spmv(op, xd, y_ref, P=P)
    torch.cuda.synchronize()
    allocations = lambda: torch.cuda.memory_stats().get("allocation.all.allocated", 0)
    before = allocations()                  # (allocation events of torch's allocator so far)
    # straight through the C ABI: descriptors, device pointers, stream
    arr = nb._pack([op])
    rc = nb.lib().nacho_spmv_static(C.cast(arr, C.c_void_p), C.c_void_p(xd.data_ptr()),
                                    C.c_void_p(y_new.data_ptr()), nb.dtype_code(xd.dtype), P,
                                    C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, nb.status_string(rc)
    torch.cuda.synchronize()
    assert allocations() == before
    a, b = y_ref.cpu().numpy(), y_new.cpu().numpy()
    assert not np.isnan(b).any()
    assert np.array_equal(a.view(np.uint8), b.view(np.uint8))


def test_two_calls_in_a_row_second_smaller():
    big = workloads.config(2, scale=0.05)
    small = workloads.config(1)
    print("static spmv: config2@0.05 then config1", flush=True)
    _both(big["A"], big["x"], 0)
    _both(small["A"], small["x"], 0)
    _both(small["A"], small["x"], 37)
    A32 = dict(small["A"], val=small["A"]["val"].astype(np.float32))
    _both(A32, small["x"].astype(np.float32), 0)


def test_too_large_is_refused_before_any_launch():
    small = workloads.config(1)
    op, xd = csr_operand(small["A"]), dev(small["x"])
    y = torch.full((small["A"]["n_rows"],), 7.0, dtype=torch.float64, device="cuda")
    P = nb.static_scratch_bytes() // 8          # 36 bytes per partition cannot fit
    with pytest.raises(nb.NachoError) as e:
        nb.nacho_spmv_static(op, xd, y, P=P)
    assert e.value.status == -6
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())
