"""MI355X-native batch step of a memory-based temporal-interaction-graph model (libtig).

`tig` is the ctypes binding over the C ABI declared in include/tig.h; `build` compiles the HIP
sources in csrc/ into libtig.so for gfx950.
"""
from . import tig  # noqa: F401

__all__ = ["tig"]
