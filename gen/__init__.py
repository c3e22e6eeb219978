"""Seeded synthetic input generators (shared by the CPU checker's tests and the GPU path's tests)."""
from . import prng, workloads  # noqa: F401
