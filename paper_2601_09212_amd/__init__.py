"""MI355X-native verify-and-resample step of annealed relaxed speculative decoding (Cool-SD).

The work is done by the C-ABI library libcool_sd.so (hand-written HIP for gfx950, declared in
include/cool_sd.h).  `binding` is a thin ctypes layer with the same entry-point names; PyTorch
is used only for device memory and streams.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    COOL_SD_BF16, COOL_SD_EARLY_EXIT_NONE, COOL_SD_EARLY_EXIT_ROUNDS, COOL_SD_EARLY_EXIT_SEQUENCE, COOL_SD_F32, COOL_SD_FLAG_CHECK_TOKENS, COOL_SD_FLAG_EARLY_EXIT, COOL_SD_FLAG_EXACT_DRAW, COOL_SD_RESAMPLE_LANTERN, COOL_SD_RESAMPLE_OPT, COOL_SD_RESAMPLE_VANILLA, COOL_SD_SCHED_EXP,
    COOL_SD_SCHED_LINEAR, COOL_SD_SCHED_UNIFORM, CoolSDError, CoolSDParams, cool_sd_bench_read_probe, cool_sd_bench_row_stats,
    cool_sd_diagnostics, cool_sd_early_exit_form, cool_sd_resample, cool_sd_schedule, cool_sd_strerror, cool_sd_verify, cool_sd_verify_diagnostics, cool_sd_verify_noalloc, cool_sd_verify_lantern,
    cool_sd_workspace_bytes, cool_sd_workspace_init, diagnostics_workload, make_params, verify_lantern_workload,
    verify_workload)
