"""Top-K+phi residual-mass decode attention on MI355X (gfx950).

The package holds the HIP kernels and their C-ABI library (`csrc/`), a thin
ctypes binding with the same entry-point names (`binding`), the build helper
(`build`) and the seeded synthetic input generators (`inputs`).  Nothing is
loaded at import time; the binding loads the shared library on first use and
raises if it has not been built.
"""
__all__ = ["binding", "inputs", "build"]
