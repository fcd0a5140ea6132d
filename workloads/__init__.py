"""Seeded synthetic inputs for the latent-KV attention path.

This package only draws random numbers and arranges them into the shapes the
benchmark configurations name. It holds none of the method's arithmetic (no
factorisation, projection, softmax or scheduling), so both the CPU oracle's
tests and the GPU path's tests can take their inputs from it without sharing
any computation.
"""
from .generators import (  # noqa: F401
    CONFIGS,
    Workload,
    adaptive_ranks,
    bf16_bits_to_f64,
    direct_latent,
    f64_to_bf16_bits,
    hidden_states,
    planted_weight,
    random_orthonormal,
    round_to_bf16,
)
