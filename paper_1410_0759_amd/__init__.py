"""igconv: implicit-GEMM convolution forward for MI355X (gfx950).

Thin ctypes binding of ``libigconv.so`` (C ABI declared in ``include/igconv.h``).
Every arithmetic step runs in the library's HIP kernels; this package only marshals
arguments.  There is no CPU fallback: if the library is missing, loading fails.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
