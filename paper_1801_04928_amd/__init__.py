"""Leapfrogging backpropagation for one MI355X: Python binding of liblf.so.

The binding marshals arguments only; every step of the pass runs in the HIP
kernels of the library.  PyTorch is used for device memory and streams.
"""
from .binding import (  # noqa: F401
    LF_OK, LF_EINVAL, LF_ESTATE, LF_ENOMEM, LF_EHIP, LF_EUNSUPPORTED,
    LF_F32, LF_BF16, LF_COST_QUADRATIC,
    LF_SCHED_AUTO, LF_SCHED_STREAMS, LF_SCHED_PERSISTENT, LF_SCHED_REDUNDANT, LF_SCHED_FUSED, LF_DEBUG_CHAIN_ONLY,
    LfError, lib, library_path,
    lf_workspace_bytes, lf_create, lf_workspace_bytes_widths, lf_create_widths,
    lf_set_params, lf_set_grad_buffers, lf_set_schedule, lf_set_debug_flags, lf_set_cost_scale, lf_set_sgd, lf_set_master_weights,
    lf_forward, lf_backward_leapfrog, lf_backward_leapfrog_noalloc, lf_noalloc_scratch_limit, lf_grads, lf_activations, lf_schedule_worker, lf_algorithm1_owner,
    lf_last_error, lf_destroy,
    LeapfrogNet,
)
