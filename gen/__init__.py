"""Seeded synthetic workloads for CSD verification (inputs only).

This package produces target-logit rows and draft tokens with the shapes and
statistics of the verification workloads; it holds none of the verification
arithmetic and is imported by both the CPU oracle's tests and the GPU tests.
"""
from .workload import (  # noqa: F401
    CONFIGS,
    WorkloadConfig,
    Workload,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    pack_pair,
)
