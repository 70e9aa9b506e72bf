"""MI355X-native fp64 GEMM (C += A*B, row-major) behind a C-ABI library.

`gemm_f64` and friends in `binding` marshal arguments to libgemm_f64.so, whose
kernels are hand-written HIP for gfx950; `synth` generates the seeded inputs
used by the tests and the benchmark.  Importing the package loads nothing
native; the first call does, and fails loudly if the library is not built.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "binding"]
__version__ = "0.1.0"
