"""MI355X-native KV-slab decode attention (hand-written HIP behind a C ABI).

``binding`` mirrors include/fineserve.h one to one; the compute runs entirely in
libfineserve.so.
"""
from .binding import *  # noqa: F401,F403
from . import binding  # noqa: F401
