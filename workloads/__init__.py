"""Seeded synthetic inputs for the operator workloads (no operator arithmetic here)."""
from . import rng, configs  # noqa: F401
