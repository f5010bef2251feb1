"""MustDrop token-reduction hot path for AMD MI355X (gfx950).

Thin binding over the C ABI in ``include/mustdrop.h`` (``libmustdrop.so``, hand-written HIP).
PyTorch is used for device memory and streams only; every step of the path runs in the library's
kernels.  There is no CPU fallback: if the library is missing, calls raise.
"""
from .binding import (  # noqa: F401
    BF16, F32, FILTER_BUDGET, FILTER_THRESHOLD, MustDropError,
    decode_workspace, encode_workspace, library, library_path, prefill_workspace,
    mustdrop_decode_append, mustdrop_decode_evict, mustdrop_decode_keep, mustdrop_encode_merge, mustdrop_encode_merge_adaptive,
    mustdrop_encode_merge_noalloc, mustdrop_prefill_filter,
    KvLayout, mustdrop_decode_append_strided, mustdrop_decode_evict_strided, mustdrop_decode_keep_strided,
    mustdrop_prefill_filter_strided,
)

__all__ = [
    "BF16", "F32", "FILTER_BUDGET", "FILTER_THRESHOLD", "MustDropError",
    "library", "library_path", "encode_workspace", "prefill_workspace", "decode_workspace",
    "mustdrop_encode_merge", "mustdrop_prefill_filter", "mustdrop_decode_evict", "mustdrop_decode_append",
    "mustdrop_decode_keep", "mustdrop_encode_merge_adaptive", "mustdrop_encode_merge_noalloc",
    "KvLayout", "mustdrop_prefill_filter_strided", "mustdrop_decode_evict_strided", "mustdrop_decode_append_strided",
    "mustdrop_decode_keep_strided",
]
