"""Hooked paged attention for MI355X: attention-mass probing and steering kernels.

Submodules are imported on demand: ``workloads`` (seeded inputs, no arithmetic)
and ``binding`` (ctypes front end of the HIP library, which raises if the
library has not been built).
"""
__all__ = ["workloads", "binding"]
