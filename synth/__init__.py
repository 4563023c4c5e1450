"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU path's tests and benchmark."""
from . import rng, workloads  # noqa: F401
