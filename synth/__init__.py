"""Seeded synthetic inputs for the RNN-T greedy-decoding hot path.

The package only draws random numbers, solves for steering frames from the
weights (adversarial.py) and lays arrays out; it contains none of the decoder's
arithmetic.  Both the CPU oracle and the HIP path consume the
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
    round_to_bf16,
    round_to_e4m3,
    with_bf16_streamed_weights,
    with_fp8_streamed_weights,
    with_streamed_weights,
)

from .adversarial import PATTERNS, emit_mask, make_adversarial, steer_frames

__all__ = [
    "PATTERNS", "emit_mask", "make_adversarial", "steer_frames",
    "Stream", "uniform", "normal", "randint",
    "ModelDims", "Model", "Workload", "CONFIGS",
    "make_model", "make_inputs", "make_workload", "param_count",
    "round_to_bf16", "round_to_e4m3", "with_bf16_streamed_weights", "with_fp8_streamed_weights", "with_streamed_weights",
]
