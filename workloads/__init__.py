"""Seeded synthetic inputs (layer-size tables and gradient generators).

Shared by the tests of the HIP path and of the CPU oracle; contains no part of
the method itself.
"""
from .gradients import GradientSource, Workload, inject_ties, layer_blocks, scaled, workloads  # noqa: F401
