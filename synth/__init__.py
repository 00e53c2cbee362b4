"""Seeded synthetic inputs for the Judge-Decoding verification head.

This package only *draws inputs*.  It contains none of the verification
arithmetic (no softmax, no accept rule, no residual, no inverse CDF), so both the
float64 oracle and the HIP library can consume its arrays without sharing any
code of the method itself.
"""

from .configs import CONFIGS, RMS_EPS, VerifyShape, make_inputs, bf16_bits_from_f32, f32_from_bf16_bits

__all__ = ["CONFIGS", "RMS_EPS", "VerifyShape", "make_inputs", "bf16_bits_from_f32", "f32_from_bf16_bits"]
