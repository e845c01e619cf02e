"""Ozaki-scheme DGEMM for one MI355X (gfx950): FP64 matrix product from FP8 / FP16 matrix-unit GEMMs.

The product is a C-ABI HIP library (csrc/, declared in include/ozaki_dgemm.h); `binding` exposes its entry
points to Python unchanged, `device` holds torch-based helpers for device buffers (memory and streams
only), `inputs` the seeded synthetic matrices of the benchmark configurations.
"""
from . import binding, inputs  # noqa: F401

__all__ = ["binding", "inputs"]
