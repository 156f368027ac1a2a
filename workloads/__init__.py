"""Seeded synthetic gradient generators shared by the tests, the benchmark and the smoke check.

This package holds input recipes only: no hashing, partitioning, bitmap or aggregation arithmetic
lives here.  Both the CPU oracle and the GPU library consume what it produces.
"""
from .generators import (  # noqa: F401
    Workload,
    WORKLOADS,
    MINI_WORKLOADS,
    get_workload,
    worker_sparse,
    dense_from_sparse,
    zipf_cdf,
)
