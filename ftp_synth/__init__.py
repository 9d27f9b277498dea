"""Seeded synthetic inputs and workload tables shared by the tests and the benchmark."""
from . import rng, configs  # noqa: F401
