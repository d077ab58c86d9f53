"""Seeded synthetic-input generators shared by the tests, the bench and the oracle's callers.

This package holds no arithmetic of the denoising method: only a counter-based Gaussian
generator, bf16 rounding helpers and the shapes of the benchmark workloads.
"""
from .rng import (fnv1a64, gaussian, gaussian_bf16, round_bf16, bf16_bits, bits_to_f32,  # noqa: F401
                  PHI64)
from .workloads import (CONFIGS, ENCODERS, DECODERS, VIDEO_DECODERS, make_requests, default_sigmas, make_inputs,  # noqa: F401
                        make_params, make_tokens)
