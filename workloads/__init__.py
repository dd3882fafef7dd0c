"""Seeded synthetic workloads: parameter-list shapes and value generators.

Shared by the tests, the benchmark and the smoke check to feed BOTH the CPU
oracle and the HIP library with the same bits.  This package holds no
arithmetic of the optimizer itself: it only names tensor shapes and draws
random numbers (conversions to BF16 are torch's).
"""
from .shapes import ParamSpec, flat_tensor, gpt2_small, resnet50, llama31_8b, llama31_8b_flat, odd_sizes  # noqa: F401
from .generate import (theta0, grad_bf16, tensor_sigma, seed_for, to_bits_u16,  # noqa: F401
                       from_bits_bf16, random_state)
