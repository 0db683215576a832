"""Seeded synthetic models and inputs for transformer-verification workloads.

This module holds no arithmetic of the verification method: it only draws
random fp32 arrays (weights, embeddings, token ids) with the shapes of the
five benchmark configurations.  Both the CPU oracle and the HIP path consume
exactly the same fp32 arrays, so weight rounding is never a parity term.
"""
from .configs import CONFIGS, EncoderConfig, Workload, get_workload, scaled
from .generate import make_model, make_tokens, make_positions

__all__ = [
    "CONFIGS", "EncoderConfig", "Workload", "get_workload", "scaled",
    "make_model", "make_tokens", "make_positions",
]
