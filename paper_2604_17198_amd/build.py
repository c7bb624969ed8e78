"""Builds libnacho.so (HIP, gfx950 only) in-tree with hipcc.

The library is compiled here, ahead of time, so that it travels with the source
tree; nothing is JIT-compiled at import.  `python -m paper_2604_17198_amd.build`
rebuilds it unconditionally.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libnacho.so")
# the same sources with -DNACHO_INSTRUMENT: every executing wavefront logs what it did (benchmarks, balance tests)
LIB_INSTR = os.path.join(PKG, "libnacho_instr.so")

SOURCES = ["api.hip", "partition.hip", "spmv.hip", "spmm.hip", "spadd.hip", "remap.hip", "validate.hip", "probe.hip"]

FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # packed fp32 arithmetic is switched off for every device function
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _hipcc() -> str:
    for c in ("/opt/rocm/bin/hipcc", "hipcc"):
        if os.path.sep not in c or os.path.exists(c):
            return c
    return "hipcc"


def _compile(job) -> str:
    src, instrumented = job
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + (".instr.o" if instrumented else ".o"))
    extra = ["-DNACHO_INSTRUMENT"] if instrumented else []
    cmd = [_hipcc(), *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def sources_present() -> list[str]:
    return [s for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]


def _link(objs, lib):
    tmp = lib + f".{os.getpid()}.tmp"
    cmd = [_hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    os.replace(tmp, lib)


def build(jobs: int = 8, instrumented: bool = True) -> str:
    """Compiles libnacho.so and (unless instrumented=False) libnacho_instr.so."""
    os.makedirs(OBJ, exist_ok=True)
    srcs = sources_present()
    work = [(s, False) for s in srcs] + ([(s, True) for s in srcs] if instrumented else [])
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, work))
    _link(objs[:len(srcs)], LIB)
    if instrumented:
        _link(objs[len(srcs):], LIB_INSTR)
    return LIB


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(ROOT, "include", "nacho.h")]
    return any(os.path.getmtime(d) > t for d in deps)


if __name__ == "__main__":
    print(build(instrumented="--fast" not in sys.argv))
