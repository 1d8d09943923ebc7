"""Seeded synthetic inputs: graphs, partitions, features, upstream gradients.

This package only draws random structure and random numbers.  It holds none of
the method's arithmetic (no quantiser, no normalisation weights, no
aggregation): both the CPU oracle's tests and the HIP path's tests take their
inputs from here and do everything else on their own side.
"""
from .graphs import (  # noqa: F401
    er_edges,
    rmat_edges,
    Partition,
    partition_by_range,
    loopback_mirror,
)
from .configs import CONFIGS, WorkloadSpec, build_workload, scaled  # noqa: F401
