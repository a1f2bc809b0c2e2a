"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU path's tests/bench.
Holds data generation only: no aggregation, combination or reordering arithmetic."""
from . import graphs, tensors, configs  # noqa: F401
