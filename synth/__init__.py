"""Seeded synthetic Q/K/V generators (inputs only; none of the method's arithmetic lives here)."""
from .workloads import CONFIGS, Workload, make_head, make_workload, hilbert_order  # noqa: F401
