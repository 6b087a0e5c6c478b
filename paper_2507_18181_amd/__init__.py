"""MI355X-native tree verification for SpecASR-style speculative decoding.

``binding``  -- ctypes view of the C ABI in include/specasr.h (libspecasr.so, HIP/gfx950).
``runtime``  -- PyTorch device-memory plumbing around it (imported on demand; needs torch).
``build``    -- hipcc build of the library.
"""
from . import binding  # noqa: F401

__all__ = ["binding"]
