"""MI355X-native per-stage training step (forward, backward, fp32 gradient accumulation, AdamW
on the data-parallel shard) behind the C-ABI library libstage.so.  This package is only the
ctypes binding: every step of the path runs in the library's HIP kernels."""
from .binding import (  # noqa: F401
    Stage, Ministages, ministages_query, StageError, lib, make_config, query, layout, fit_linear, loss_scale_update, ops, wgrad_parts, wgrad_parts_cut, wgrad_parts_scratch_bytes, STAGE_OK, STAGE_ERR_ARG, STAGE_ERR_STATE,
    STAGE_ERR_WORKSPACE, STAGE_ERR_BUDGET, STAGE_ERR_DEVICE,
)
