"""Seeded synthetic inputs for the BNS-GCN partition step.

This package only *draws inputs*: graphs, partitions, features, labels and
initial weights.  It holds none of the method's arithmetic (no hashing, no
sampling, no normalisation, no layer maths) and is imported by the tests and
the benchmark, which hand the same arrays to the CPU oracle and to the HIP
library.
"""
from .partition import Partition, partition_from_entries, partition_of_global_graph
from .graphs import sbm_graph, chung_lu_partition0
from .workloads import Workload, CONFIGS, make_workload, SAMPLING_SEED

__all__ = [
    "Partition", "partition_from_entries", "partition_of_global_graph",
    "sbm_graph", "chung_lu_partition0",
    "Workload", "CONFIGS", "make_workload", "SAMPLING_SEED",
]
