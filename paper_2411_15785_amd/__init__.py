"""libbct: the Bounded-Cache Transformer decode path on AMD MI355X (gfx950).

HIP kernels and the C ABI live in csrc/ (declared in include/bct.h); this
package is the thin ctypes binding over the built libbct.so.
"""
from .binding import (BCT_BF16, BCT_ERR_BUFFER_TOO_SMALL, BCT_ERR_HIP, BCT_ERR_INVALID_ARG,  # noqa: F401
                      BCT_ERR_MISALIGNED, BCT_ERR_STATE, BCT_ERR_UNSUPPORTED, BCT_F32,
                      BCT_MK_PER_SEQUENCE, BCT_OK, BCT_STEP_STREAMING, BctCache, BctError, bct_cache_desc, bct_cache_init,
                      bct_cache_query, bct_last_error, bct_plan_query, bct_strerror, lib, make_desc)
