"""paper_2012_00596_amd — Python binding of libnpas (HIP, gfx950).

Argument marshalling only: every step of the sparse-inference path runs inside
the C-ABI library declared in include/npas.h.  PyTorch is used by callers for
device memory and streams; this module only takes `data_ptr()`s.
There is no CPU fallback: if the library is not built, importing works but the
first call raises.
"""
from .binding import *  # noqa: F401,F403
from .binding import build, lib  # noqa: F401
