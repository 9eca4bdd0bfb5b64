"""Seeded synthetic inputs shaped like the paper's streaming workloads.

Serves both the oracle-side tests and the HIP-side tests/benchmark.  Holds none of the
method's arithmetic: only shapes, seeds, random draws and dtype rounding.
"""
from .configs import (  # noqa: F401
    Workload,
    WORKLOADS,
    get,
    seed_for,
    randn,
    make_qkv,
    make_evicted,
    rope_tables,
    frame_grid,
    to_f64,
)
