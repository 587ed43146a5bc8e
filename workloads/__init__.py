"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package only draws random inputs (token streams, bf16 K/V/q bit patterns,
weight tables).  It contains none of the method's arithmetic and imports neither
the oracle nor the HIP binding.
"""
from .synth import (  # noqa: F401
    CONFIGS,
    Workload,
    WorkloadConfig,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    make_workload,
    make_tokens,
    make_kv,
    make_queries,
    make_drifting_queries,
    make_qwin,
    extra_queries,
)
