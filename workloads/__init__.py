"""Seeded synthetic inputs shaped like the paper's click-log workloads.

This package only *generates inputs* (tables, id streams, frequency ranks,
gradients).  It contains none of the cache method's logic and is the single
thing the CPU oracle's tests and the GPU path's tests/bench have in common.
"""
from .gen import (  # noqa: F401
    Workload,
    make_workload,
    table_values,
    fill_host_table,
    zipf_positions,
    log_uniform_cardinalities,
    CONFIG_NAMES,
)
