"""MI355X-native fold step of KV-Fold: thin Python binding over the C-ABI library libkvfold.so.

Every step of the path (append, chunk-prefix attention, split merge) runs in the HIP kernels of
the library; this package only marshals arguments.  PyTorch is used by callers for device
memory and streams.
"""
from .binding import (  # noqa: F401
    KVFOLD_BF16, KVFOLD_F32, KvFoldError, KvFoldCache, TUNE_SPLITS, TUNE_UNITS_PER_WAVE, TUNE_PAIR_UNITS, TUNE_FUSED_APPEND, lib_path, load_library,
    kvfold_cache_bytes_required, kvfold_cache_create, kvfold_cache_destroy, kvfold_cache_length, kvfold_cache_plan, kvfold_plan_for, kvfold_cache_profile_begin, kvfold_cache_profile_end,
    kvfold_cache_set_length, kvfold_cache_set_storage_roundtrip, kvfold_cache_set_tuning, kvfold_cache_truncate, kvfold_cache_view, kvfold_config_t, kvfold_last_hip_error,
    kvfold_status_string, kvfold_step, kvfold_step_ex, kvfold_step_rope, kvfold_step_window, kvfold_step_noalloc, kvfold_plan_t, kvfold_measure_peaks,
)
