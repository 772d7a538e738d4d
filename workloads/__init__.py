"""Seeded synthetic workloads: stage shapes and input generators.

This package holds shape records and random draws only.  None of the method's
arithmetic (layer math, gradients, optimizer) lives here, so both the CPU
oracle's tests and the HIP path's tests can be fed from it without the two
sharing any computation.
"""
from .configs import StageConfig, CONFIGS, get_config  # noqa: F401
from .inputs import StageInputs, make_inputs, round_bf16, round_f16  # noqa: F401
