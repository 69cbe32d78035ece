"""CPU oracle of the AcceRL actor forward pass.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package;
the HIP library and its Python binding never do, and nothing here imports them.
`oracle.c` holds one direct-loop C function per layer type; `forward.py` strings them into
a network in the order the layer list gives; `ptq.py` is the post-training quantizer and the
channel pruner that produce a student policy from fp32 weights.
"""
from .clib import build, lib  # noqa: F401
from . import layers  # noqa: F401
from .forward import forward_float, forward_int8, forward_mixture  # noqa: F401
from .ptq import quantize_policy, prune_policy, QuantPolicy, derived_constants  # noqa: F401
