"""Seeded synthetic input generators shared by the oracle tests, the GPU parity tests and bench.py.

This package draws random inputs only (token ids, Q/K/V/dO tensors, KV caches, flags). It holds
none of the method's arithmetic: no mask, no softmax, no compaction. Both the CPU oracle and the
HIP path consume what it returns as plain numpy arrays.
"""
from .generators import (  # noqa: F401
    SEPARATOR_IDS,
    VOCAB,
    AttnConfig,
    CacheConfig,
    CONFIGS,
    bf16_round,
    make_token_ids,
    make_qkv,
    make_dO,
    make_cache,
    cache_to_ring,
    cache_from_ring,
    config_inputs,
    small_variant,
)
