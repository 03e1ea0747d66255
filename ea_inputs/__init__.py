"""Seeded synthetic KV-cache inputs shared by the tests, the bench and the oracle checks.

This package only *draws inputs* (random pre-RoPE activations, the rotary embedding that
turns them into cached keys / window queries, rounding to the storage dtype).  It holds none
of the compression method's arithmetic (no statistics, no scores, no selection), and neither
the oracle nor the HIP library imports it: callers pass its arrays to both.
"""
from .configs import CacheConfig, CONFIGS, get_config          # noqa: F401
from .host import (make_layer, bf16_bits_from_f64, f64_from_bf16_bits,  # noqa: F401
                   inv_freq_table, layer_seed, widen, make_block_pools, quantize_fp8)
