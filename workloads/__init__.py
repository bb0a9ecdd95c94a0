"""Seeded synthetic inputs for the five workloads.

This module serves both the CPU oracle's tests and the GPU path's tests and
benchmark.  It holds none of the method's arithmetic: only shapes, seeded random
draws (numpy PCG64) and the flat parameter layout used to hand weights over.
"""
from .configs import WORKLOADS, Workload, make_inputs, xavier_mlp, random_involution, uniform_memory, MASTER_SEED  # noqa: F401
