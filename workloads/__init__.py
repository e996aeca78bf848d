"""Seeded synthetic workloads (inputs only; none of the method's arithmetic lives here)."""
from .synth import *  # noqa: F401,F403
from .synth import MASTER_SEED, Workload  # noqa: F401
