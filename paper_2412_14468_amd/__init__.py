"""MI355X-native HashAttention decode path (arxiv 2412.14468, section 4).

`binding` holds the ctypes front end of libhashattn.so (hand-written HIP for
gfx950 behind a C ABI, see include/hashattn.h); `build` compiles it.
"""
from .binding import (Context, HashAttnError, KvCache, Mlp, load, hashattn_gather_attend_noalloc,  # noqa: F401
                      OK, INVALID_ARG, UNSUPPORTED, SCRATCH_TOO_SMALL, HIP_ERROR)
