"""libdz: base GEMM + selective batched matmul (SBMM) over compressed deltas on AMD MI355X.

Thin ctypes binding of the C ABI in include/dz.h: the functions below have the C names and only
marshal arguments (tensor -> pointer, shape -> ints, torch stream -> hipStream_t).  Every step of
the computation runs in the HIP kernels of libdz.so; torch is used for device memory and streams
only.  There is no fallback: if libdz.so has not been built, importing the binding raises.
"""
from .binding import *          # noqa: F401,F403
from .binding import __all__    # noqa: F401
