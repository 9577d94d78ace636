"""MI355X-native boundary layout transform (forward materialise / backward
route) of heterogeneous-parallel multimodal training: a C-ABI library of HIP
kernels (libhp.so) plus this thin binding."""
from .binding import (HpError, Plan, hp_backward, hp_backward_accumulate, hp_forward, hp_forward_static, hp_get_option, hp_plan_create,
                      hp_plan_create_batched, hp_plan_create_host, hp_plan_create_joined, hp_plan_tune, hp_probe_stream, hp_probe_stream_ex,
                      hp_forget_tuned_shapes, hp_release_cached_memory, hp_profile_enable, hp_profile_read, hp_set_option, hp_version)
from .workloads import Grid, TokenMap

__all__ = ["Grid", "TokenMap", "Plan", "HpError", "hp_plan_create", "hp_plan_create_host", "hp_plan_create_batched", "hp_plan_create_joined", "hp_plan_tune", "hp_probe_stream", "hp_probe_stream_ex", "hp_release_cached_memory", "hp_forget_tuned_shapes",
           "hp_forward", "hp_forward_static", "hp_backward", "hp_backward_accumulate", "hp_set_option", "hp_get_option", "hp_profile_enable", "hp_profile_read", "hp_version"]
