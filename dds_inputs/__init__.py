"""Seeded synthetic workloads shared by the CPU oracle's tests and the HIP path's tests.

This package holds DATA only: network descriptions (lists of op records), module
boundaries, and counter-seeded generators for mini-batches and initial weights.
It contains none of the training method's arithmetic (no forward, backward,
schedule or update code) and imports neither the oracle nor the HIP binding.
"""
from .configs import Workload, workload, WORKLOAD_NAMES  # noqa: F401
from .gen import make_batch, make_params, param_shapes  # noqa: F401
