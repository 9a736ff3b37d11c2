"""Seeded synthetic inputs for the selective-recompute prefill path.

This package only draws random numbers and shapes them (hidden rows, weights,
auxiliary attention blocks, chunk layouts).  It contains none of the method's
arithmetic, so both the CPU oracle's tests and the HIP path's tests can take
their inputs from it without sharing any of the code under test.
"""
from .configs import ModelShape, Workload, CONFIGS, get_workload  # noqa: F401
from . import gen  # noqa: F401
