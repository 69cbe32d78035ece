"""Seeded synthetic inputs and network shapes for the AcceRL actor-forward path.

This package is the only code shared by the CPU oracle and the HIP library's
tests/bench.  It holds no arithmetic of the method itself: only a counter-based
random generator, the recipes that turn it into observations, uniforms, initial
weights and recurrent state, and the layer lists of the benchmark networks.
"""
from .rng import BASE_SEED, STREAM, u64, uniform01, normal, randint  # noqa: F401
from .nets import (  # noqa: F401
    Net, conv, dense, maxpool, resblock, relu, flatten, lstm,
    mlp, nature_cnn, impala_cnn, paper_small_cnn, param_shapes, feature_dim, trace_shapes,
)
from .data import (  # noqa: F401
    init_params, make_obs_f32, make_frames_u8, make_uniforms, make_done, make_hc,
    make_logits_pair, make_trajectory,
)
from .configs import CONFIGS, get_config  # noqa: F401
