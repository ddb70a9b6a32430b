"""MI355X-native per-processor lowered-einsum path of a mesh-laid-out Transformer layer.

Thin ctypes binding over libmtf.so (C ABI in include/mtf.h).  Every step of the path runs in
the library's HIP kernels; Python only marshals arguments.  PyTorch supplies device memory
and the stream.  There is no fallback: if the library is missing, importing `binding` fails.
"""
from .binding import *  # noqa: F401,F403
