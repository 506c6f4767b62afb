"""Seeded synthetic inputs for the ADORE decode hot path.

This package holds shapes and random numbers only: none of the method's
arithmetic lives here.  Both the CPU oracle's tests and the HIP path's
harness draw their inputs from it, so the two sides see identical bytes.
"""
from .synthetic import Workload, WORKLOADS, workload, round_bf16, SyntheticInputs, DeviceNormals  # noqa: F401
