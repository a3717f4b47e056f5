"""Seeded synthetic workloads: variable lists and input generators.

This package holds shapes and random-number plumbing only.  None of the
method's arithmetic (layout equations, optimizer steps) lives here, so both
the CPU oracle's tests and the HIP path's tests may draw inputs from it.
"""
from .configs import CONFIGS, Workload, get_workload  # noqa: F401
from .gen import normal_f32, random_bits_u32, variable_inputs  # noqa: F401
