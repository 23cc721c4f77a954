"""Seeded synthetic inputs for the CALS hot path.

This package only *generates data* (tensors, starting points, model lists).  It holds none of
the method's arithmetic (no MTTKRP, no Gram, no solve, no fit) and is the only code that both
the CPU oracle's tests and the HIP path's tests / benchmark use.
"""
from .configs import CONFIGS, WorkloadConfig, get_config  # noqa: F401
from .generators import (  # noqa: F401
    make_tensor,
    make_inits,
    make_models,
    uniform_factors,
    random_tensor,
    low_rank_tensor,
    low_rank_tensor_device,
)
