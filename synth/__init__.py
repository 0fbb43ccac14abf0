"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package draws graph structure and random values only.  Normalisation weights,
aggregation, transforms and gradients are NOT computed here: the oracle and the HIP
library each do that on their own.
"""
from . import graphs, values  # noqa: F401
from .configs import CONFIGS, Workload, make_graph  # noqa: F401
