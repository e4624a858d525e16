"""dfq on MI355X: the int8 / power-of-two-scale quantized convolution path of
arXiv 1805.07941 as hand-written HIP kernels for gfx950 behind a C-ABI library
(include/dfq.h, libdfq.so), with a thin ctypes binding.

``from paper_1805_07941_amd import binding`` loads the library and fails loudly when
it has not been built (``python -m paper_1805_07941_amd.build``); there is no CPU path.
"""
from . import binding  # noqa: F401

__all__ = ["binding"]
