"""MI355X-native AllGather-GEMM consumer and GEMM-ReduceScatter reducer.

Thin ctypes binding over libagg.so (include/agg.h).  Every step of the hot path
runs in the library's HIP kernels; this package only marshals arguments.
There is no CPU fallback: importing `binding` fails if the library is not built.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
