"""MI355X-native pack/unpack of strided MPI derived datatypes (TEMPI, arXiv 2012.14363).

The product is the C-ABI library `libtp_pack.so` (see include/tp_pack.h); this
package is its build script and a ctypes binding with the same names.
"""
from . import binding  # noqa: F401
from .binding import *  # noqa: F401,F403
