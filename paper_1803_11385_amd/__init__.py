"""hch: the hot path of H-CNN (PSH-based sparse 3-D convolution and pooling) on MI355X.

Thin ctypes binding over the C-ABI shared library libhch.so (sources in csrc/,
declarations in include/hch.h).  Every step of the path runs in the library's HIP
kernels; this package only marshals arguments.  There is no CPU fallback: if the
library is missing, importing `binding` raises.
"""
from .binding import *  # noqa: F401,F403
from . import binding as _binding

__all__ = list(_binding.__all__)
