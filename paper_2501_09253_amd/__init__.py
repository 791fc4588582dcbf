"""MI355X-native patched denoising block (PatchedServe hot path): thin binding over libpserve.so."""
from .binding import (  # noqa: F401
    Plan, Block, Cache, PserveError, lib, library_path, set_kernel_mode, profile_enable, profile_read, profile_select, profile_sample,
    F32, BF16, STAGE_KIND, TABLES, SLOT_H1, SLOT_R, SLOT_K, SLOT_V, SLOT_Y, Resample, DOWN2, UP2,
    latency_predict, latency_fit, slack, schedule, probe_mfma_bf16, probe_mfma_mix, probe_copy,
)
