"""MI355X-native PacTrain compression path: mask -> compress -> sum over workers -> decompress.

The work is done by libpactrain.so (hand-written HIP kernels behind the C ABI of
include/pactrain.h).  This package only marshals arguments: torch tensors supply device memory
and streams.  There is no CPU or eager fallback; a missing library is an error.
"""
from .binding import (  # noqa: F401
    PAC_BF16, PAC_F32, PacError, PacContext, library_path, load_library,
    pac_build_mask, pac_compress, pac_create, pac_debug_set_candidate_capacity, pac_decompress,
    pac_destroy, pac_keep_count, pac_last_error, pac_mask_words, pac_reduce_local,
    MaskTracker, pac_decompress_update, pac_mask_equal, pac_mask_from_nonzero, pac_tracker_create,
    pac_tracker_destroy, pac_tracker_update, pac_absmax, pac_ternarize, pac_ternary_reduce_local,
    pac_step_fused, pac_device_status, pac_debug_set_scan_spin_limit, pac_mask_from_nonzero_noalloc, PAC_DEV_SCAN_STALLED, PAC_DEV_COUNT_MISMATCH,
    PAC_DEV_META_MISMATCH, PAC_DEV_RETRY_TAKEN, PAC_DEV_SLOW_PATH, PAC_DEV_ERROR_MASK, PAC_TABLE_SLOTS,
)
