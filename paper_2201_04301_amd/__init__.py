"""G-CADA hot path for AMD MI355X: hand-written HIP kernels behind a C-ABI (include/gcada.h).

``binding`` mirrors the C entry points one to one; ``run`` holds a small convenience wrapper that
keeps the torch tensors (device memory) alive around a context.
"""
from . import binding  # noqa: F401  (fails loudly when libgcada.so is not built)
from .run import Gcada  # noqa: F401
