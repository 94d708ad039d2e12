"""Seeded synthetic workloads for batched VLA policy inference.

This package only *draws inputs*: model shapes, weight tensors, patch
embeddings, instruction ids, ragged lengths and Gumbel noise.  It contains none
of the policy's arithmetic (no norm, attention, matmul, softmax or
de-tokenisation), so that the CPU oracle and the HIP library can both be fed
from it without sharing any code of the method itself.
"""
from .configs import PolicyShape, Workload, WORKLOADS, get_workload  # noqa: F401
from .generate import (  # noqa: F401
    bf16_bits_from_f32, f32_from_bf16_bits, tensor_rng, weight_names,
    make_weights, make_observations, make_gumbel, weight_shape, make_value_weights,
)
