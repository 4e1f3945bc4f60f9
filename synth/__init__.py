"""Seeded synthetic inputs for the paged-KV decode / KV-reclamation path.

This package only *produces inputs* (pool geometry, block tables, context
lengths, bf16 bit patterns).  It holds none of the method's arithmetic: no
attention, no relocation planning, no table rewriting.  Both the CPU oracle
tests and the GPU tests draw their inputs from here so that the two sides see
identical bits.
"""
from .workload import (  # noqa: F401
    Geometry,
    Workload,
    PoolState,
    WORKLOADS,
    workload,
    build_state,
    hash_bf16_bits,
    hash_bf16_bits_torch,
    pool_bits_for_blocks,
    fill_pool_torch,
    fill_pool_range_torch,
    query_bits,
    poison_unused_slots,
    unused_slot_spans,
    sample_ctx_len,
    BF16_NAN_BITS,
)
