"""MI355X-native stage training for FTPipeHD: thin Python binding over the C-ABI
library libftp_hip.so (hand-written HIP kernels for gfx950).  PyTorch is used by
callers only for device memory and streams."""
from .binding import (  # noqa: F401
    FtpError, lib, last_error,
    model_create, model_destroy, model_num_units, model_unit_in_shape, model_unit_param_count,
    model_unit_bn_channels, stage_create, stage_destroy, stage_import_weights, stage_export_weights,
    stage_export_grads, stage_export_momentum, stage_export_bn_stats, stage_export_conv_output, stage_export_bn_batch_stats, stage_forward, stage_loss, softmax_ce_static, STATIC_LOSS_MAX_BATCH,
    stage_snapshot_weights, stage_aggregate_weights, stage_copy_units, stage_timing, stage_timing_read, stage_device_bytes, STAGE_RECOMPUTE, redistribution_plan, renumber_workers, repartition_due, repartition_capacities, stage_backward, stage_update, profile_layers, solve_partition,
    estimate_capacity, ktrace_begin, ktrace_end, calibration_copy, diag_fail_next_launch_plan, F32, BF16,
)
from . import models  # noqa: F401
