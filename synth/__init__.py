"""Seeded synthetic inputs (model shapes, weights, token ids) shared by the
CPU oracle's tests and the HIP library's tests and benchmark.

This package holds no decoder arithmetic: it only names shapes and draws
random numbers.  Neither the oracle nor the HIP path lives here.
"""
from .workloads import (  # noqa: F401
    CONFIGS,
    Workload,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    make_tokens,
    make_weights,
    scaled_workload,
    sub_slice_of,
    tp_slice,
    workload,
)
