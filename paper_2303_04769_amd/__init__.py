"""MI355X-native (gfx950) implementation of the SMaLL abstract-layer hot path.

`binding` is a thin ctypes layer over libsmall_hip.so (the C ABI of include/small.h):
argument marshalling only, every step of the path runs in the HIP kernels. PyTorch is
used for device memory and streams. There is no CPU fallback: loading fails loudly when
the library is missing.
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
