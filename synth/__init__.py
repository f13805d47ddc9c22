"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

Holds generators only (random graphs, features, weights, labels).  Neither the HIP library
nor the CPU oracle is imported here, and none of the method's arithmetic lives here.
"""
from . import configs, graphs, model, rng  # noqa: F401
from .configs import WORKLOADS, Workload, get_workload  # noqa: F401
