"""Helpers for the GPU parity tests: move generated inputs to the device and
wrap them in the binding's operand descriptors.  No arithmetic of the method."""
from __future__ import annotations

import numpy as np
import torch

from paper_2604_17198_amd import binding as nb


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


def csr_operand(A):
    return nb.csr(dev(A["pos"]), dev(A["crd"]), A["n_rows"], A["n_cols"], dev(A["val"]))


def dcsr_operand(A):
    return nb.dcsr(dev(A["pos0"]), dev(A["crd0"]), dev(A["pos1"]), dev(A["crd1"]),
                   A["n_rows"], A["n_cols"], dev(A["val"]))


def vector_operand(v):
    return nb.vector(dev(v["i"]), v["extent"], dev(v["v"]))


def parts_to_numpy(parts):
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in parts.items()}
