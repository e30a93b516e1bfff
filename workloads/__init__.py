"""Seeded synthetic workloads for the neighbourhood-attention hot path.

This package only draws random inputs and arranges them (coordinates, storage
rounding, ordering of tokens into equal-size clusters).  It contains none of
the method's arithmetic (no distances-to-neighbours, no softmax, no attention)
and is the one module both the CPU oracle's tests and the HIP path's tests use.
"""
from .synth import (  # noqa: F401
    CONFIGS,
    WorkloadConfig,
    bf16_round,
    make_coords,
    make_features,
    make_workload,
    morton_cluster_order,
    random_neighbours,
)
