"""Seeded synthetic inputs shared by the tests, the benchmark and the CPU oracle.

This package only produces inputs (graphs, initial tables, workload descriptions).
It holds none of the training method's arithmetic: no hashing of negatives, no
scores, no loss, no optimiser.
"""

from .graphs import (  # noqa: F401
    Workload,
    WORKLOADS,
    rows_per_partition,
    generate_edges,
    bucket_edges,
    init_tables,
    scaled,
)
