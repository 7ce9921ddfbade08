"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package holds workload *descriptions* (sizes) and seeded random *inputs* only.
It contains none of the method's arithmetic (no Philox, no MLP, no GAE, no PPO).
"""
from .synthetic import (  # noqa: F401
    PPOConfig,
    CONFIGS,
    get_config,
    param_count,
    make_model_params,
    make_env_matrices,
    make_initial_state,
    make_rollout_batch,
)
