"""MI355X-native frequency-aware software cache for large embedding tables (after arXiv:2208.05321).

The product is the C-ABI library `libfreqcache.so` (hand-written HIP for gfx950, see include/freqcache.h).
This package is its thin Python binding: argument marshalling only, PyTorch supplies device memory and
streams.  There is no CPU fallback: without the built library or without a GPU the calls raise.
"""
from .binding import (  # noqa: F401
    FreqCache,
    FreqCounter,
    table_reorder,
    FreqCacheError,
    load_library,
    FC_WARM,
    FC_TRANSMIT_STAGED,
    FC_EVICT_DMA,
    STAT_FIELDS,
)
