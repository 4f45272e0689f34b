"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package holds input generation only: random tensors, planted structure and
budget draws.  None of the method's arithmetic (pooling, scoring, selection,
attention, partitioning) lives here, and it imports neither the oracle nor the
HIP binding.
"""
from .synth import (  # noqa: F401
    CONFIGS,
    Workload,
    bf16_bits_from_f32,
    f32_from_bf16_bits,
    layer_budgets,
    make_workload,
    make_custom,
    one_kv_head_per_query_head,
    take_heads,
)
