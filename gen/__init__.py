"""Seeded synthetic workload generators (inputs only; no method arithmetic)."""
from .workloads import *  # noqa: F401,F403
from .workloads import Workload, F32, BF16  # noqa: F401
