"""MI355X (gfx950) shared-pool paged decode attention with balloon bookkeeping.

Thin Python face of libprismkv.so (C-ABI in include/prism_kv.h).  The package
fails loudly when the HIP library is missing: there is no CPU fallback.
"""
from .binding import PrismKV, PKV_BF16, PKV_E4M3, lib_path, arbitrate_requests, place_models  # noqa: F401
