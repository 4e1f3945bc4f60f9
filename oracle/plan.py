"""Split of one decode batch into work items and bounded slices (test oracle).

The paper requires offline compute to stop within a bounded, sub-millisecond
time (Section 2.3, Challenge 1; Section 4.1) without waiting for kernel, layer
or iteration boundaries.  This build meets that bound cooperatively: the
attention of one layer is cut into slices that each read at most `slice_bytes`
of KV, and a yield lands between two slices.  This module states which work
goes into which slice.

work item  = (sequence, kv_head, first_block_index, n_tokens): a run of at most
             `chunk_tokens` consecutive context tokens of one KV head.
order      = sequence-major, then chunk, then kv head (the heads of one chunk
             sit next to each other in memory, so neighbours in launch order
             read neighbouring addresses).
slice      = maximal run of consecutive items whose K+V bytes sum to at most
             `slice_bytes`; a slice always holds at least one item.
"""
from __future__ import annotations

import numpy as np


def attention_plan(ctx_len, num_kv_heads: int, head_dim: int, block_tokens: int,
                   chunk_tokens: int, slice_bytes: int):
    """Returns (work int32 [n_items, 4], slice_start int32 [n_slices + 1])."""
    if chunk_tokens <= 0 or chunk_tokens % block_tokens:
        raise ValueError("chunk_tokens must be a positive multiple of the block size")
    work = []
    for s, n in enumerate(int(v) for v in ctx_len):
        if n < 1:
            raise ValueError("context length must be at least 1")
        first = 0
        while first < n:
            ntok = min(chunk_tokens, n - first)
            for h in range(num_kv_heads):
                work.append((s, h, first // block_tokens, ntok))
            first += chunk_tokens
    token_bytes = 2 * head_dim * 2  # one K row and one V row, bf16
    starts = [0]
    acc = 0
    for i, (_, _, _, ntok) in enumerate(work):
        b = ntok * token_bytes
        if i > starts[-1] and acc + b > slice_bytes:
            starts.append(i)
            acc = 0
        acc += b
    starts.append(len(work))
    return (np.asarray(work, dtype=np.int32).reshape(-1, 4),
            np.asarray(starts, dtype=np.int32))
