"""PolarQuant KV-cache hot path for MI355X: thin Python binding over libpolarquant.

The C ABI is declared in ``include/polarquant.h``; this package only marshals
arguments (tensor pointers, sizes, the current HIP stream).  Every step of the
path runs in the library's kernels; there is no Python or CPU fallback.
"""
from .binding import (  # noqa: F401
    PQ_BF16, PQ_F32, PQ_KEY, PQ_VALUE, TILE_TOKENS, TILE_CODE_BYTES, TILE_RADII, RECORD_BYTES,
    PolarQuantError, Context, library, pq_status_string, profile_begin, profile_end,
    GeneralFormat, general_encode, general_decode, general_attn_decode,
)
