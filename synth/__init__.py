"""Seeded synthetic inputs for the relay-race hot path.

This package holds input generation only: a counter-based random number
generator, storage-type rounding, and the workload shapes.  It contains none
of the model's arithmetic, so both the CPU oracle's tests and the HIP path's
tests may draw their inputs from it without sharing any computation.
"""
from .generator import (  # noqa: F401
    ModelConfig,
    Workload,
    WORKLOADS,
    make_weights,
    make_batch,
    make_lengths,
    normal,
    uniform_int,
    round_to_bf16,
)
