"""Seeded synthetic inputs shared by the HIP path's tests, the oracle's tests and bench.py."""
from . import prng, configs  # noqa: F401
