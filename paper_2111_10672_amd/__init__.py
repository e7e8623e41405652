"""SPB worker step for MI355X: thin Python binding over the C ABI in include/spb.h.

Every step of the path runs in the HIP kernels of libspb.so; this package only marshals
arguments.  torch is used for device memory and streams.
"""
from .binding import (  # noqa: F401
    SpbError, SpbModel, lib, library_path,
    spb_model_create, spb_model_destroy, spb_num_units, spb_param_count, spb_param_info,
    spb_bind_params, spb_bind_grads, spb_workspace_size, spb_forward, spb_backward_truncated,
    spb_grad_buffers, spb_zero_absent_grads, spb_set_kernel_timing, spb_read_kernel_timing, spb_replay_kernel,
    spb_last_error, desc_from_config, spb_worker_depth, spb_aggregate_update, spb_schedule_tasks,
    spb_forward_static, SPB_STATIC_WORKSPACE_BYTES, spb_unit_io, SPB_VIEW_CALLER_INPUT, SPB_VIEW_NONE,
)
