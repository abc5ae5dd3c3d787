"""MI355X-native lifetime-aware tensor offloading for LLM training (hot path of arXiv 2506.06472).

The product is libteraio.so (C ABI in include/teraio.h, HIP kernels for gfx950); this package is
the thin ctypes binding plus the in-tree build driver.
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
