"""Seeded synthetic inputs shaped like the paper's long-context attention workloads.

This package holds input generation only: random draws, bf16 rounding of the drawn
values, shape tables and row-sample selection.  None of the method's arithmetic
(scores, softmax, merge) lives here, so the CPU oracle's tests and the HIP path's
tests can both take their inputs from it without sharing any computation.
"""
from .synthetic import (  # noqa: F401
    CONFIGS,
    AttnConfig,
    MergeConfig,
    bf16_bits_to_f32,
    bf16_bits_to_f64,
    f32_to_bf16_bits,
    make_merge_partials,
    make_qkv_bits,
    sample_rows,
)
