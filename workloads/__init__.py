"""Seeded synthetic inputs for the backup-worker Sync-SGD step.

This package only draws random numbers and describes configurations.  It
holds none of the method's arithmetic (no selection, no reduction, no
optimizer update), so both the CPU oracle's tests and the HIP path's tests
may feed from it without sharing any logic.
"""
from .configs import CONFIGS, StepConfig, get_config, scaled_config  # noqa: F401
from .gen import (  # noqa: F401
    BLOCK,
    arrival_times,
    arrival_matrix,
    grad_block,
    grad_row,
    grad_columns,
    grad_matrix,
    theta0,
    tensor_sizes,
    tensor_layout,
    lr_at,
    row_scale_vector,
    n_blocks,
    block_columns,
)
