"""libabft: checksum-protected GEMM for MI355X (gfx950).

The work is done by hand-written HIP kernels in ``csrc/`` behind the C ABI
declared in ``include/abft.h``; ``binding`` only marshals arguments.
"""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
