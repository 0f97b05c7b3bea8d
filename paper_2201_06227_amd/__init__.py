"""MI355X-native plasticity-evaluation path of Egeria (arXiv 2201.06227).

The product is `libegeria.so` (hand-written gfx950 kernels behind the C-ABI of
include/egeria.h).  `binding` is the thin ctypes layer over it; PyTorch is used
for device memory and streams only.
"""
from . import _build  # noqa: F401

__all__ = ["binding", "_build"]
