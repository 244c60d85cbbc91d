"""Seeded synthetic inputs shared by the HIP path's harness and by the CPU oracle's tests.

This package holds no arithmetic of the method itself: it only draws Q/K/V tensors with
the shapes and statistics of the paper's workloads (Experiments, "Models": 21 x 3600 and
33 x 3600 video tokens per head) and the random index draws used to seed k-means.
"""
from .generators import (  # noqa: F401
    Workload,
    WORKLOADS,
    get_workload,
    make_qkv,
    kmeans_init_indices,
    budget_pairs,
)
from .sampling import structural_rows  # noqa: F401
