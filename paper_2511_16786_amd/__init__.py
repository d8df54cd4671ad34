"""MI355X-native prefill-time KV-cache compression (score -> allocate -> select+gather).

The package is a thin binding over libflashcache.so (hand-written HIP for gfx950).
"""
from . import binding
from .binding import (  # noqa: F401
    FC_PATH_AUTO, FC_PATH_DENSE, FC_PATH_FFT, Compressor, FcKvDesc, FlashCacheError,
    allocate, cutoff_r, decode_attention, decode_attention_paged, decode_attention_static,
    decode_static_scratch_bytes, describe, lowpass_energy, prepare, resolve_path, score, score_layer, select_gather, select_gather_paged,
    total_budget,
    workspace_bytes, workspace_error,
)
