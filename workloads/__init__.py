"""Seeded synthetic inputs and the five workload shapes.

This package holds no arithmetic of the SBP method: it only makes input
tensors.  Both the CPU oracle's tests and the HIP path's tests / bench take
their inputs from here; neither the oracle nor the HIP package imports it.
"""
from .generate import (SEED_BASE, normal, uniform, to_bf16_bits, bf16_bits_to_f32,  # noqa: F401
                       pattern_u16)
from .configs import CONFIGS  # noqa: F401
