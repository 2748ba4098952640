"""MI355X-native per-worker GraphSAGE-mean training step (hand-written HIP for gfx950).

The compute lives in libsdt.so (sources under csrc/, C ABI in include/sdt.h);
this package only marshals arguments.  There is no CPU fallback.
"""
from .binding import *  # noqa: F401,F403
from .binding import lib, Csr, Block, SdtError, Timing, make_model, ws_view  # noqa: F401
