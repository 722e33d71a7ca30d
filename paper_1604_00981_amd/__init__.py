"""bsgd: the parameter-side step of synchronous SGD with backup workers
(Algorithm 4 of "Revisiting Distributed Synchronous SGD") as hand-written HIP
kernels for MI355X behind a C ABI (include/bsgd.h), plus this thin binding."""
from .binding import (  # noqa: F401
    BSGD_OK, BSGD_ERR_ARG, BSGD_ERR_TOO_FEW, BSGD_ERR_HIP, BSGD_ERR_SCRATCH, BSGD_STATIC_SCRATCH_BYTES,
    BSGD_MAX_WORKERS, BSGD_MAX_TENSORS, bsgd_step_noalloc,
    BSGD_SGD, BSGD_MOMENTUM, BSGD_RMSPROP_MOM,
    BsgdError, bsgd_hyper, bsgd_tensor, bsgd_select_opts, make_select_opts,
    bsgd_select_ex, bsgd_step_ex, bsgd_last_kept_count,
    load_library, make_hyper, make_tensors, alloc_workspace,
    bsgd_select_first_n, bsgd_reduce_update, bsgd_step, bsgd_workspace_bytes,
    bsgd_last_status, bsgd_last_selection, bsgd_last_clip, bsgd_calibration_copy, bsgd_set_tuning, bsgd_set_table_mode, bsgd_num_shapes, bsgd_get_shape, bsgd_last_launch_count, bsgd_debug_chunk_runs, bsgd_set_fused_selection, bsgd_last_step_fused_selection, bsgd_version, strerror,
    bsgd_last_gradient_count, bsgd_precombine, bsgd_yardstick_streams,
    bsgd_straggler_workspace_bytes, bsgd_kth_arrival_times, bsgd_time_to_converge,
)
