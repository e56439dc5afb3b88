"""MI355X (gfx950) library for CKKS-encrypted ternary matrix multiplication.

`binding` is a ctypes layer over libensi_hip.so (see include/ensi.h); the
package holds no arithmetic of its own.
"""
from . import binding  # noqa: F401
from .binding import Context, EnsiError  # noqa: F401
