"""A2SGD (two-level gradient averaging, arXiv 2006.07405) per-step hot path for one MI355X: HIP kernels behind a
C ABI (include/a2sgd.h) and a ctypes binding of the same names."""
from .binding import (A2SGD_MAX_WORKERS, A2SGD_MODE_ALG1_LITERAL, A2SGD_MODE_RETAINED_ERROR, A2SGD_OK,
                      A2SGD_ERR_INVALID_ARG, A2SGD_ERR_ALIGNMENT, A2SGD_ERR_DEVICE, A2SGD_ERR_NOMEM,
                      A2SGD_ERR_WORKSPACE_TOO_SMALL, A2SGD_ERR_WORKSPACE_STATE, A2SGD_ERR_SCRATCH_LIMIT,
                      A2SGD_STATIC_SCRATCH_BYTES, A2sgdError,
                      Plan, WorkerStats, a2sgd_plan, a2sgd_workspace_bytes, a2sgd_plan_blocks_per_worker, a2sgd_plan_single_launch_cell,
                      a2sgd_workspace_check, a2sgd_device_info, a2sgd_export_local_means, a2sgd_import_global_means,
                      alloc_workspace, a2sgd_local_averages, a2sgd_global_average, a2sgd_apply_and_update_error,
                      a2sgd_step, a2sgd_step_static, a2sgd_read_stats, a2sgd_export_mask, a2sgd_dense_step,
                      a2sgd_apply_and_update_error_replicas, a2sgd_step_replicas, a2sgd_dense_step_replicas,
                      a2sgd_replica_drift, a2sgd_lazy_reset, a2sgd_lazy_step, a2sgd_lazy_local_averages, a2sgd_lazy_apply, a2sgd_lazy_materialize, a2sgd_selftest_barrier, a2sgd_workspace_init, a2sgd_read_segment_stats, raw,
                      LIB_PATH)
