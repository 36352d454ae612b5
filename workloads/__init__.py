"""Seeded synthetic workloads shared by the tests, the CPU oracle and the HIP path.

This package only draws random inputs (hidden states, weights, token ids,
lengths, rewards, logZ) and rounds them to the storage type.  It contains none
of the method's arithmetic, so both the oracle and the GPU library may be fed
from it without sharing code with each other.
"""
from .configs import Workload, CONFIGS, get_config
from .gen import (
    bf16_bits_from_f32,
    f32_from_bf16_bits,
    as_f64,
    lengths,
    rewards,
    log_z,
    tokens,
    matrix,
    matrix_rows,
    hidden,
    weight,
    perturbed_weight,
    sample_valid_rows,
    synthetic_logprobs,
    synthetic_upstream_grad,
    STREAM_H,
    STREAM_W,
    STREAM_W_OLD,
    STREAM_W_REF,
)

__all__ = [
    "Workload", "CONFIGS", "get_config",
    "bf16_bits_from_f32", "f32_from_bf16_bits", "as_f64",
    "lengths", "rewards", "log_z", "tokens",
    "matrix", "matrix_rows", "hidden", "weight", "perturbed_weight",
    "sample_valid_rows", "synthetic_logprobs", "synthetic_upstream_grad",
    "STREAM_H", "STREAM_W", "STREAM_W_OLD", "STREAM_W_REF",
]
