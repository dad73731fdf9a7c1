"""MI355X-native HeatKV hot path: thin ctypes binding over libheatkv.so.

Every step of the path (calibration masses, schedule construction, cache
append/compaction, attention over the ragged cache) runs inside the library;
this package only marshals arguments.  PyTorch tensors are used as device
memory handles and for the current HIP stream.
"""
from .binding import (  # noqa: F401
    HeatKVError,
    KV_FP8_E4M3,
    KV_NATIVE,
    Plan,
    Shape,
    VARIANT_BINARY,
    VARIANT_BINARY_NAIVE,
    VARIANT_HEATKV,
    VARIANT_NAIVE,
    calibrate,
    heatkv_accumulate_beta,
    heatkv_append_scale,
    heatkv_attend_append_scale,
    heatkv_attend_scale,
    heatkv_build_schedule,
    heatkv_build_schedule_kv,
    heatkv_calibrate,
    heatkv_calibrate_accumulate,
    heatkv_calibrate_scales_accumulate,
    heatkv_calibrate_static,
    heatkv_head_scores,
    heatkv_load_schedule,
    heatkv_load_schedule_kv,
    heatkv_rank_dispersion,
    library_path,
)
