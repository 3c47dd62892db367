"""Seeded synthetic inputs shared by the CPU oracle and the HIP path.

Nothing in here is part of the method (no sampling, no cache policy, no gather): it only
manufactures graphs, feature tables and seed batches of the shapes the paper trains on.
Integer-only torch ops are used so that the same seed gives the same arrays on the CPU and
on the GPU.
"""
from .configs import CONFIGS, Workload, make_workload  # noqa: F401
from .rmat import rmat_csr  # noqa: F401
