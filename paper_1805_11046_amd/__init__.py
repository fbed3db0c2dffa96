"""8-bit training hot path (quantized back-propagation + Range BN) on MI355X.

`paper_1805_11046_amd.binding` mirrors the C ABI of libq8t.so (include/q8t.h); importing it
fails if the library has not been built (there is no fallback path).
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
