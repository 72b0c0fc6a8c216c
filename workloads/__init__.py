"""Seeded synthetic inputs for the LightKV compression step.

This module only draws random tensors and describes shapes and schedules
(grid, window counts per axis, token targets).  It contains none of the
method's arithmetic: no similarity, no attention weight, no selection, no
merge.  The HIP path and the CPU oracle are both fed from here, by the tests
and by the benchmark, and neither of them imports the other.
"""
from .synthetic import (  # noqa: F401
    CONFIGS,
    Workload,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    make_workload,
    make_custom,
)
