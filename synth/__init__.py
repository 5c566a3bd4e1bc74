"""Seeded synthetic inputs (weights, queries, masks) shared by the CPU oracle and the HIP path.

This package holds input generation only: no part of the model forward, the sampler or the
log-softmax lives here.
"""
from .inputs import (  # noqa: F401
    ModelConfig,
    Workload,
    WORKLOADS,
    make_weights,
    make_queries,
    make_random_responses,
    make_tensor,
    boost_eos,
    boost_eos_bias,
    round_to_bf16,
    bf16_bits,
    weight_names,
    weight_shape,
)
