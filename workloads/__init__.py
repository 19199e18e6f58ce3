"""Seeded synthetic KV-cache workloads (inputs only).

This package draws the Q/K/V tensors that both the CPU oracle and the HIP
library are run on.  It holds no part of the compression method: nothing here
computes attention, scores, ranks, budgets or gathers.
"""
from .gen import (  # noqa: F401
    WorkloadConfig,
    get_config,
    seq_lens,
    budget_for,
    make_layer,
    f32_to_bf16_bits,
)
