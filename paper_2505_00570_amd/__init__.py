"""MI355X-native FreqKV KV-cache compression: thin ctypes binding over libfreqkv (HIP, gfx950)."""
from .binding import (  # noqa: F401
    AttendPlan, BF16, F32, FLAG_DENSE, FLAG_DROPPING, FLAG_NO_RESCALE, FLAG_RETAIN_HIGH, FLAG_SINGLE_FOLD, FLAG_TWO_LEVEL_FOLD, FreqKVError, Layout, Plan, Profile,
    PrefillPlan, attend_decode, attend_decode_noalloc, attend_decode_ragged, attend_plan, attend_prefill, attend_prefill_plan,
    calibrate_copy, calibrate_mfma, compress, compress_ragged, last_error, lib_path, load, noalloc_scratch_bytes, plan, power_spectrum, prepare, profile_enable, profile_read,
    shutdown, status_string, version,
)
