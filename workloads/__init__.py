"""Seeded synthetic workloads (data only; see synth.py)."""
from .synth import SPECS, WorkloadSpec, make, trace, profile, configs, slos, class_edges, checksum  # noqa: F401
