"""Seeded synthetic inputs shared by the HIP path's tests/benchmark and the CPU oracle.

Holds input recipes only (random data, labels, straggler masks); none of the
method's arithmetic lives here.
"""
from .workloads import *  # noqa: F401,F403
