"""Seeded synthetic inputs for the cached-prefill path.

This module is the only code shared by the CPU oracle's tests and the HIP path's
tests/benchmark.  It draws lengths, values and page tables; it contains none of
the method's arithmetic (no RoPE, no attention, no truncation rule, no packing).
"""
from .workloads import (  # noqa: F401
    CONFIGS,
    Workload,
    bf16_bits_to_f64,
    draw_block_table,
    draw_lengths,
    draw_values_bf16,
    f32_to_bf16_bits,
    make_workload,
)
