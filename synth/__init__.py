"""Seeded synthetic inputs for the stage workloads.  Serves both the CPU oracle
and the HIP path; holds none of the method's arithmetic (only random draws,
bf16 rounding of the drawn values, and index slicing of tensor-parallel shards).
"""
from .stage_inputs import *  # noqa: F401,F403
