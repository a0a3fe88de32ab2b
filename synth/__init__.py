"""Seeded synthetic inputs for the RNN-T greedy-decoding hot path.

This module only draws random numbers and lays them out; it contains none of
the decoder's arithmetic.  Both the CPU oracle and the HIP path consume the
arrays produced here, so neither depends on the other.

Random numbers come from a counter-based generator written out below
(splitmix64 finaliser over a 64-bit counter), so the bytes do not depend on any
library's RNG version.
"""
from .rng import Stream, uniform, normal, randint
from .workloads import (
    ModelDims,
    Model,
    Workload,
    CONFIGS,
    make_model,
    make_inputs,
    make_workload,
    param_count,
)

__all__ = [
    "Stream", "uniform", "normal", "randint",
    "ModelDims", "Model", "Workload", "CONFIGS",
    "make_model", "make_inputs", "make_workload", "param_count",
]
