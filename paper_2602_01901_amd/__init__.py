"""Lazy Attention with the layer-shared Q Cache for AMD MI355X (gfx950).

The product is the C-ABI library declared in include/qcache.h (HIP kernels in csrc/); this
package is its thin Python binding plus `Session`, a convenience wrapper that uses PyTorch only
to own device memory and the stream.
"""
from .binding import *  # noqa: F401,F403
from .binding import EXPORTED, LIB_PATH, QcError, load_library, make_config
from .session import Session

__all__ = ["Session", "QcError", "load_library", "make_config", "EXPORTED", "LIB_PATH"]
