"""MI355X (gfx950) implementation of the smoothed W8A8 expert FFN of HAQ
(arXiv 2508.07329, Section III.B): a C-ABI HIP library (libhaq.so, see
include/haq.h) and this thin ctypes binding.  PyTorch is used only to own device
memory and streams; every step of the path runs in the library's kernels.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
