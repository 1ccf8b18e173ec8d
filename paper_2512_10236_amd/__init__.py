"""MI355X-native finer-grain compute/communication overlap: all-gather -> GEMM (and GEMM ->
reduce-scatter data movement) with copy-engine transfers and hand-written gfx950 MFMA kernels.

The product is ``libficco.so`` (``csrc/``, C ABI in ``include/ficco.h``); this package is its
ctypes binding. PyTorch is not imported here: callers use it for device memory and streams.
"""
from .binding import *  # noqa: F401,F403
from . import binding as _b

__all__ = [n for n in dir(_b) if n.startswith(("ficco_", "FICCO_"))] + ["FiccoError", "SCHEDULE_NAMES", "load",
                                                                          "library_path", "EXPORTS"]
