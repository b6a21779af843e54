"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

Nothing in this package performs any step of the BitStack method: it only draws
random weights, scales, activations and (for the large shapes) random residual
blocks with a stated magnitude profile.
"""
from .synth import (  # noqa: F401
    BASE_SEED,
    CONFIGS,
    LLAMA3_8B_LINEARS,
    activations,
    column_scales,
    dense_weight,
    llama3_8b_layer_shapes,
    rng_for,
    synthetic_blocks,
    variable_n_loaded,
)
