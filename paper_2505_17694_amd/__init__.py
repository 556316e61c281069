"""Prefix-shared decode attention for MI355X (gfx950): Python face of libcodec.so.

``binding`` mirrors the C ABI of include/codec.h name for name; ``runtime``
adds a thin holder that keeps a plan together with the PyTorch tensors used as
its device memory.  There is no CPU fallback: without the built library the
import fails.
"""
from .binding import *          # noqa: F401,F403
from .binding import EXPORTED_SYMBOLS, LIB_PATH, CodecError
from .runtime import PlannedAttention

__all__ = ["EXPORTED_SYMBOLS", "LIB_PATH", "CodecError", "PlannedAttention"]
