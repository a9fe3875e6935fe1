"""Seeded synthetic inputs for the link-prediction training step.

This module only draws random inputs (graphs, features, weights, batches).  It
contains none of the method's arithmetic: no CSR construction, no aggregation,
no sampling of negatives, no loss.  Both the CPU oracle's tests and the HIP
path's tests/benchmarks take their inputs from here so that they see the same
bytes.
"""
from .graphs import (  # noqa: F401
    CONFIGS,
    PartitionedInputs,
    Workload,
    chung_lu_edges,
    make_partitioned,
    make_workload,
    partition_edge_lists,
    uniform_edges,
    worker_view,
)
from .model_init import init_features, init_model, to_bf16_grid  # noqa: F401
