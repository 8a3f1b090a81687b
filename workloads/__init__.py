"""Workload shapes (configs) and seeded synthetic input generators (synth)."""
from .configs import WORKLOADS, VARIANTS, Workload, MASTER_SEED  # noqa: F401
