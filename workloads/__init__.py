"""Seeded synthetic inputs for the DSV sparse-attention hot path.

This package only draws and rounds numbers.  It holds none of the method's
arithmetic (no projection, scoring, selection, softmax or gradients), so that
both the CPU oracle's tests and the HIP path's tests can take their inputs from
it without sharing any code of the method itself.
"""
from .configs import CONFIGS, WorkloadConfig, get_config  # noqa: F401
from .generator import (  # noqa: F401
    round_to_dtype,
    basis,
    head_tensors,
    predictor_weights,
    k_per_head,
    idx_offsets,
    random_subset_idx,
    progression_params,
    progression_idx_rows,
    progression_queries_of_key,
    ternary_head_tensors,
    head_tensors_smooth,
)
