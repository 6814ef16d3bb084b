"""Seeded synthetic workloads for the XOR-encrypted sparse quantized weight path.

This package only *makes inputs*: weight draws, the pruning mask, the binary-coded
bit-planes with their per-row scales, the XOR-network matrix M and the activation
matrix X.  It contains none of the method's arithmetic (no GF(2) product, no
encoder, no decoder, no matrix product), so both the CPU oracle's tests and the
GPU library's tests/bench may import it without sharing any code of the method.
"""
from .configs import CONFIGS, WorkloadConfig, get_config
from .generate import (
    Workload,
    bf16_bits_to_f32,
    draw_M,
    draw_W,
    draw_X,
    f32_to_bf16_bits,
    greedy_binary_code,
    magnitude_mask,
    make_workload,
    pad_columns,
    random_care_problem,
)

__all__ = [
    "CONFIGS",
    "WorkloadConfig",
    "get_config",
    "Workload",
    "bf16_bits_to_f32",
    "draw_M",
    "draw_W",
    "draw_X",
    "f32_to_bf16_bits",
    "greedy_binary_code",
    "magnitude_mask",
    "make_workload",
    "pad_columns",
    "random_care_problem",
]
