"""One GPU's share of an expert-parallel MoE layer for AMD MI355X (gfx950): hand-written HIP kernels behind a
C ABI (``include/moe355.h``) and a thin ctypes binding.  Importing the package loads nothing; the shared library
is opened on first use and its absence is an error (there is no CPU fallback)."""
from . import workloads  # noqa: F401  (pure NumPy, no GPU)

__all__ = ["workloads", "binding", "layer"]
