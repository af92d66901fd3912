"""MI355X-native quantized matrix-product path (quant_int, dot'_int, fused
epilogues) of arxiv 1805.12096.  The work is done by hand-written gfx950 HIP
kernels behind a C boundary (include/mq.h); this package is the thin binding."""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
