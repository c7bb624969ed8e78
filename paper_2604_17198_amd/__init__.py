"""MI355X-native hot path of the load-balanced sparse tensor algebra partitioner.

Sub-modules:
  workloads -- seeded synthetic input generators (no arithmetic of the method)
  build     -- compiles the HIP library (hipcc, gfx950) in-tree
  binding   -- thin ctypes binding over the C-ABI of libnacho.so

Nothing is imported eagerly: `workloads` is usable without the HIP library and
`binding` raises if the library has not been built.
"""

__all__ = ["workloads", "build", "binding"]
