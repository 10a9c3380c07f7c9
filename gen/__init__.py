"""Seeded synthetic inputs shaped like the paper's Criteo workloads.

This package only draws random inputs (table sizes, weights, index batches,
upstream gradients).  It contains none of the method's arithmetic, so both the
CPU oracle's tests and the GPU path's tests may use it without sharing any
code that computes results.
"""
from .workloads import (  # noqa: F401
    CONFIGS,
    Workload,
    cardinalities,
    make_workload,
    make_tables,
    index_batch,
    grad_dyadic,
    grad_normal,
    DENSE_CONFIGS,
    make_dense_model,
    dense_batch,
    split_batch,
)
