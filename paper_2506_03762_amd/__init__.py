"""AhaKV eviction hot path for AMD MI355X (gfx950).

``binding`` marshals torch tensors into the C ABI of ``include/aha.h``
(libaha.so, hand-written HIP kernels); ``synth`` draws the seeded synthetic
workloads; ``build`` compiles the library in-tree.
"""
from . import synth  # noqa: F401  (numpy only)

__all__ = ["synth", "binding", "build"]
