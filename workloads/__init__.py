"""Seeded synthetic inputs shaped like the paper's workloads (Table II).

This package only *draws inputs*: feature matrices, labels and the item / level /
tie hypervector tables that the library and the test oracle both receive as
arguments.  It contains none of the method's arithmetic (no quantiser, no binding,
no bundling, no distances) and imports neither the HIP binding nor the oracle.
"""
from .synthetic import Workload, make_workload, CONFIGS, pack_bits_lsb  # noqa: F401
