"""Fused Mixture-of-Experts layer forward for AMD Instinct MI355X (gfx950).

`synthetic` draws seeded workloads; `binding` is the ctypes front end of the
HIP library (built by `build.py`).  Importing this package loads neither.
"""
