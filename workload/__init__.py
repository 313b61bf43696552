"""Seeded synthetic workloads shared by the tests, the oracle's callers and the benchmark."""
from . import configs, synth  # noqa: F401
