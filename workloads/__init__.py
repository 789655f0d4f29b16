"""Seeded synthetic inputs for shared-prefix decode attention.

This package only *produces inputs*: request shapes, lengths, sharing
structure, block-pool free orders, and the stored Q/K/V bits (fp32, bf16 or
fp8-e4m3 codes with per-tile scales).  It contains none of the method's
arithmetic (no block allocation policy, no attention, no fp8 decode) and is the
only module imported by both the CPU oracle's tests and the HIP path's tests.
"""
from .generate import (  # noqa: F401
    CONFIG_NAMES,
    Geometry,
    PoolData,
    ScoreShape,
    Workload,
    bf16_bits_from_f32,
    chunk_prefill_workload,
    e4m3_encode,
    fill_pool,
    ideal_bytes,
    make_tree_workload,
    make_workload,
    named_chunk_prefill,
    named_tree_workload,
    named_workload,
)
