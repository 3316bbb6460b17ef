"""MI355X-native low-rank bottleneck decoder-block hot path (hand-written HIP behind a C ABI).

`paper_2512_12131_amd.binding` holds thin ctypes wrappers with the same names as the C entry
points in include/lrboost.h.  Importing this package does not load the shared library; the
first call does, and it raises if the library has not been built (no CPU fallback exists).
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
