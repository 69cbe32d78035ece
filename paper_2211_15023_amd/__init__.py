"""MI355X-native actor forward of the AcceRL paper: thin Python binding over libaccerl.so.

Everything on the path runs in the HIP kernels of csrc/; this package only marshals arguments.
PyTorch provides device memory and streams, nothing else.
"""
from .binding import (  # noqa: F401
    AccerlError, Policy, load_library, make_arch, pack_weights, pack_scales, blob_sizes,
    accerl_policy_create, accerl_policy_destroy, accerl_actor_forward, accerl_actor_forward_teacher,
    accerl_actor_forward_recurrent, accerl_actor_forward_debug, accerl_last_error,
    accerl_profile_begin, accerl_profile_end, accerl_plan_describe, accerl_monitor_kl, accerl_monitor_kl_noalloc, accerl_vtrace, accerl_distill_loss, accerl_actor_forward_mixture, accerl_mixture_alpha, accerl_probe_mfma, accerl_probe_copy, accerl_probe_empty,
    INT8, FP32, BF16, TAP_ACC, TAP_ACT, TAP_ACC_A, TAP_ACT_A,
)
