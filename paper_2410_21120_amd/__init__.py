"""MI355X-native fused multi-model CNN inference (FusedInf hot path).

The product is the C-ABI library `libfusedinf.so` (see include/fusedinf.h); this
package is a thin ctypes binding with the same entry-point names.  Every step
of the path runs in the library's HIP kernels: nothing here computes.
"""
from .binding import *  # noqa: F401,F403
