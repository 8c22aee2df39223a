"""Centroid-based semantic cache hot path (batched lookup, centroid update,
self-similarity merge) as hand-written HIP kernels for gfx950.

Sub-modules are imported on demand:

* ``paper_2508_18736_amd.siso``      - thin binding over the C-ABI library
  (``libsiso.so``); raises at import time if the library has not been built.
* ``paper_2508_18736_amd.workloads`` - seeded synthetic input generators
  (numpy only; no arithmetic of the method itself).
"""

__all__ = ["siso", "workloads"]
