"""Seeded synthetic inputs (graphs, partitions, features, drift streams) shared by
the CPU oracle's tests and the GPU path's tests and benchmark. Input data only."""
from . import rng, graphs, features, configs  # noqa: F401
