"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This package only draws random numbers and lays them out in flat buffers with
the shapes and value distributions of the five workloads.  It contains none of
the optimizer step's arithmetic and imports neither the GPU library nor the
CPU oracle; both consume the bytes produced here.
"""
from .configs import WORKLOADS, Workload  # noqa: F401
