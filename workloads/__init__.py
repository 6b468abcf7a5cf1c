"""Seeded synthetic inputs for the decode-step path: model shapes, weight and
KV bit patterns, block tables.

This package only produces data (shapes, random bf16 bit patterns, integer
tables).  It contains none of the transformer arithmetic: both the CPU oracle
and the HIP path consume its arrays as inputs.
"""
from .configs import CONFIGS, ModelConfig, Workload, WORKLOADS  # noqa: F401
from .generate import (  # noqa: F401
    bf16_bits_from_f32, f32_from_bf16_bits, normal_bf16, make_weights,
    fill_kv_pool, initial_tokens, pool_shape, BF16_NAN_BITS,
)
from .blocktable import build_block_tables, draw_contexts, BlockLayout  # noqa: F401
