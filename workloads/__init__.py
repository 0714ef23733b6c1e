"""Seeded synthetic inputs for the tests and the benchmark (no method arithmetic)."""
from . import gen, configs  # noqa: F401
