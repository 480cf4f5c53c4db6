"""LUT-multiplier conv2d / dense for AMD MI355X (gfx950).

The package holds the HIP kernels behind a C ABI (``csrc/``), a ctypes binding with
the same entry-point names (``binding``), the build helper (``build``) and the seeded
synthetic-input generators (``inputs``).  Nothing here falls back to a CPU path: the
binding raises when the HIP library is missing.

Sub-modules are imported on demand so that ``inputs`` can be used without the HIP
library being present.
"""

__all__ = ["binding", "build", "inputs"]
