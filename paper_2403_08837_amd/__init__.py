"""libcdp: single-GPU hot path of Cyclic Data Parallelism on MI355X (gfx950).

The product is the C-ABI shared library built from ``csrc/`` (declared in
``include/cdp.h``); ``binding`` is its thin ctypes wrapper.
"""
from . import binding  # noqa: F401
from .binding import Trainer, CdpError  # noqa: F401
