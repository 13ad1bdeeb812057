"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package holds shapes, workload descriptions and random-number draws only.
None of the method's arithmetic (norms, projections, attention, rotation,
scoring, selection) lives here.
"""
from .workloads import (  # noqa: F401
    ModelShape,
    Workload,
    WORKLOADS,
    budget_to_k,
    make_weights,
    make_hidden,
    make_influence,
    make_block_table,
    ragged_lengths,
    round_to_bf16,
    stream_rng,
)
