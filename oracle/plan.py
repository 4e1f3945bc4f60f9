"""Split of one decode batch into work items and bounded slices (test oracle).

The paper requires offline compute to stop within a bounded, sub-millisecond
time (Section 2.3, Challenge 1; Section 4.1) without waiting for kernel, layer
or iteration boundaries.  This library meets that bound cooperatively: the
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

A context length of 0 stands for a sequence that is not in the batch (a request
that was evicted and sent back to the waiting state, Section 5, "Sub-layer
memory reclamation"): it contributes no work.
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
        if n < 0:
            raise ValueError("context length must not be negative")
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


def prefill_plan(ctx_len, q_len, num_q_heads: int, num_kv_heads: int, head_dim: int, block_tokens: int,
                 chunk_tokens: int, slice_bytes: int):
    """Work split of a causal prefill step (the newest q_len[s] tokens of every sequence).

    tile  = up to 128 // GP consecutive new positions of one sequence (GP = query heads per kv
            head, rounded up to a power of two): (sequence, first q row, first position, positions);
            q rows are packed sequence after sequence.
    item  = (tile, kv_head, first_block_index, n_tokens): a chunk of at most chunk_tokens of the
            tokens the tile can see (0 .. its last position); order tile, chunk, kv head.
    slice = maximal run of items with at most slice_bytes of K+V (at least one item).
    Returns (work [n_items,4], slice_start, tiles [n_tiles,4], tile_base [n_tiles+1]).
    """
    if chunk_tokens <= 0 or chunk_tokens % 32:
        raise ValueError("chunk_tokens must be a positive multiple of 32")
    group = num_q_heads // num_kv_heads
    gp = 1
    while gp < group:
        gp *= 2
    qp = 128 // gp
    work, tiles, tile_base = [], [], []
    row = 0
    for s, (n, ql) in enumerate(zip((int(v) for v in ctx_len), (int(v) for v in q_len))):
        if ql < 1 or n < ql:
            raise ValueError("need 1 <= q_len <= context length")
        t = 0
        while t * qp < ql:
            n_pos = min(qp, ql - t * qp)
            pos0 = n - ql + t * qp
            tile_base.append(len(work))
            tiles.append((s, row + t * qp, pos0, n_pos))
            visible, first = pos0 + n_pos, 0
            while first < visible:
                for h in range(num_kv_heads):
                    work.append((len(tiles) - 1, h, first // block_tokens, min(chunk_tokens, visible - first)))
                first += chunk_tokens
            t += 1
        row += ql
    tile_base.append(len(work))
    token_bytes = 2 * head_dim * 2
    starts, acc = [0], 0
    for i, w in enumerate(work):
        b = w[3] * token_bytes
        if i > starts[-1] and acc + b > slice_bytes:
            starts.append(i)
            acc = 0
        acc += b
    starts.append(len(work))
    return (np.asarray(work, dtype=np.int32).reshape(-1, 4), np.asarray(starts, dtype=np.int32),
            np.asarray(tiles, dtype=np.int32).reshape(-1, 4), np.asarray(tile_base, dtype=np.int32))
