"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This package produces *data only*: counter-based pseudo-random integers, weight tensors,
token templates, retrieval pools and contexts. It contains none of the method's
arithmetic (no suffix matching, no transformer maths, no acceptance rule), so both the
oracle and the GPU path may be fed from it without sharing any implementation.
"""
from .rng import hash_u64, uniform_tokens, approx_normal_f32, round_to_bf16_f32, bf16_bits  # noqa: F401
from .model import ModelShape, SHAPES, weight_names, gen_weight, gen_all_weights  # noqa: F401
from .workload import PoolSpec, POOLS, gen_templates, gen_pool, gen_contexts, noisy_copy  # noqa: F401
