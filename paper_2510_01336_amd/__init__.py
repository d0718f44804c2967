"""MI355X (gfx950) implementation of HiSpec's k-token verification path.

The product is the C-ABI library `libhispec.so` (see include/hispec.h).  This
package is a thin ctypes binding with the same entry-point names: it only
marshals arguments.  PyTorch is used for device memory and streams.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
