"""Seeded synthetic inputs for the NetMax iteration: workload configurations,
policy matrices built from synthetic link-speed matrices, data shards and
initial parameters.

This package holds *inputs only*.  None of the method's arithmetic (peer
sampling, thresholds, gradients, mixing, consensus distance) lives here; both
the HIP library and the CPU oracle receive what these functions return as plain
arrays.
"""
from .configs import Workload, workload, WORKLOAD_NAMES, BASE_SEED, hyperparameters  # noqa: F401
from .policy import (  # noqa: F401
    policy_from_speeds,
    floor_and_renormalise,
    default_rho,
    link_speeds,
    policy_for,
    iteration_times,
    dynamic_times,
)
from .data import make_shards, init_params, f32_to_bf16_bits, bf16_bits_to_f32  # noqa: F401
