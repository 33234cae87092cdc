"""Seeded synthetic inputs for the Judge Q eviction hot path.

This package only produces inputs (soft-token queries, prefix keys/values,
budgets, ragged offsets).  It contains none of the method's arithmetic (no
softmax, pooling, selection or gather), so both the CPU oracle's tests and the
HIP path's tests/bench can draw identical bits from it.
"""
from .generate import (  # noqa: F401
    CONFIGS,
    Workload,
    bf16_bits_to_f32,
    bf16_bits_to_f64,
    f32_to_bf16_bits,
    make_workload,
    page_out,
)
