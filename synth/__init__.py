"""Seeded synthetic inputs shared by the CPU oracle and the HIP path.

This package holds no arithmetic of the method itself: it only draws random
weights and token ids of requested shapes, and knows the five workload
configurations by name.
"""
from .inputs import CONFIGS, gen_params, gen_tokens, iter_params_pooled, to_bf16_round  # noqa: F401
