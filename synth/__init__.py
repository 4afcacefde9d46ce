"""Seeded synthetic inputs for the FLy verification step.

This package holds only input generation (shapes, counter-based random
numbers, workload presets).  It contains none of the method's arithmetic and
is the one module that both the CPU oracle's tests and the HIP path's tests
draw their inputs from.
"""
from .workloads import (  # noqa: F401
    CONFIGS,
    VerifyConfig,
    hash_normal,
    hash_uniform,
    hash_tokens,
    layer_weight_shapes,
    make_weight,
    make_kv_prefix,
    make_row_temperature,
    make_first_tokens,
    make_draft_draws,
    TENSOR_IDS,
    make_hidden,
)
