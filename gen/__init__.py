"""Seeded synthetic workload generators (inputs only; no method arithmetic)."""
from .workloads import *  # noqa: F401,F403
from .workloads import Workload, F32, BF16  # noqa: F401
from .trace_inputs import trace_logits, KINDS as TRACE_KINDS  # noqa: F401
from .loss_inputs import loss_inputs  # noqa: F401
