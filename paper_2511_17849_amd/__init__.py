"""MI355X-native hot path of Pier's two-level optimizer: a C-ABI HIP library
(libpier.so, sources in csrc/, ABI in include/pier.h) and this thin ctypes binding.
There is no CPU fallback: loading fails loudly when the library has not been built."""
from .binding import (  # noqa: F401
    PierError, PierCtx, AdamwHP, OuterHP, OffloadStats,
    PIER_PHASE_WARMUP, PIER_PHASE_PIER, PIER_LOC_DEVICE, PIER_LOC_HOST_PINNED,
    pier_ctx_create, pier_ctx_destroy, pier_ctx_numel, pier_ctx_set_launch, pier_ctx_set_occupancy, pier_ctx_set_offload_writeback,
    pier_bind_replica, pier_bind_shadow, pier_bind_outer, pier_inner_adamw, pier_outer_step,
    pier_inner_adamw_clipped, pier_inner_adamw_clipped_static, pier_ctx_set_norm_fold, pier_grad_norm_last,
    pier_offload_workspace_bytes, pier_offload_stream, pier_hbm_probe, pier_hbm_probe_summary, pier_hbm_classify, pier_placement_plan,
    pier_mu_schedule, pier_outer_lr_schedule, pier_outer_schedule,
    pier_inner_lr_schedule, pier_train_step, TrainCfg, PIER_MODE_PIER, PIER_MODE_DILOCO,
    pier_last_error, pier_status_string, library_path, pier_abi_version,
)
from .hbm_arena import HbmArena, ModelBuffers  # noqa: F401
