"""Seeded synthetic workloads: chain descriptions (plain data) and input generators.

This module serves both the CPU oracle and the HIP library and therefore holds none of the
method's arithmetic: it only says which kernels a chain has, which operands they take, and how
the random tensors are drawn.  Neither `oracle/` nor the product package is imported here.
"""
from .spec import ChainSpec, KernelSpec, TensorSpec, Ref, EXT, INT, WEIGHT  # noqa: F401
from .configs import (  # noqa: F401
    BASE_SEED,
    elementwise_chain,
    decode_chain,
    refresh_stress_chain,
    large_tensor_chain,
    decode_buckets,
    bucket_sequence,
    tiny_mixed_chain,
)
from .data import (  # noqa: F401
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    draw_tensor,
    make_weights,
    make_inputs,
)
