"""MI355X-native boundary layout transform (forward materialise / backward
route) of heterogeneous-parallel multimodal training: a C-ABI library of HIP
kernels (libhp.so) plus this thin binding."""
from .binding import (HpError, Plan, hp_backward, hp_backward_accumulate, hp_forward, hp_forward_static, hp_zero_image_rows, hp_get_option, hp_plan_create,
                      hp_plan_create_batched, hp_plan_create_host, hp_plan_create_joined, hp_plan_tune, hp_probe_stream, hp_probe_stream_ex,
                      hp_forget_tuned_shapes, hp_release_cached_memory, hp_profile_enable, hp_profile_read, hp_set_option, hp_version)
from .workloads import Grid, TokenMap


def boundary_transform(plan, src_bufs, text_bufs):
    """The transform as one differentiable PyTorch operation (see autograd.py;
    imported on first use so that host-only users of the plan builder do not
    need torch)."""
    from .autograd import boundary_transform as _impl
    return _impl(plan, src_bufs, text_bufs)


__all__ = ["Grid", "TokenMap", "boundary_transform", "Plan", "HpError", "hp_plan_create", "hp_plan_create_host", "hp_plan_create_batched", "hp_plan_create_joined", "hp_plan_tune", "hp_probe_stream", "hp_probe_stream_ex", "hp_release_cached_memory", "hp_forget_tuned_shapes",
           "hp_forward", "hp_forward_static", "hp_zero_image_rows", "hp_backward", "hp_backward_accumulate", "hp_set_option", "hp_get_option", "hp_profile_enable", "hp_profile_read", "hp_version"]
