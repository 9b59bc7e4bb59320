"""Seeded synthetic inputs for the ATP hot path.

This module holds no arithmetic of the method itself: it only draws random
matrices with a prescribed singular spectrum, noise level and shape, and rounds
them to the storage type of a call.  Both the CPU oracle's tests and the HIP
path's tests/bench read the very same host buffers produced here.
"""
from .generators import (  # noqa: F401
    BASE_SEED,
    Workload,
    CONFIGS,
    config_seed,
    spectrum,
    make_X,
    make_omega,
    make_weight,
    round_to_bf16,
    round_to_dtype,
    sweep_point,
)
