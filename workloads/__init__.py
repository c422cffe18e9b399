"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

Nothing in this package performs any step of the method (no dequantization, no
masking, no index compaction, no layout permutation, no dot products): it only
draws random tensors of the documented shapes and distributions, encodes them in
the row-major *source* format that both sides take as input, and picks thresholds
as order statistics of |x|.
"""
from .synth import (  # noqa: F401
    GROUP,
    TILE_ROWS,
    CONFIG_SHAPES,
    CONFIG_SCALE_RANGE,
    KIND_WEIGHTS,
    KIND_X,
    KIND_CALIB,
    seed_for,
    make_weights,
    make_fp_weights,
    make_x,
    quantile_threshold,
    calibrated_threshold,
    make_case,
)
