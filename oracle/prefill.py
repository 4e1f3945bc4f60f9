"""fp64 causal attention of a chunk of new tokens over a paged bf16 KV cache (test oracle).

The paper names long prefills ("e.g., 32k tokens", Section 2.2; Section 5 on bursts arriving
during a long prefill iteration) as the case where coarse preemption hurts most.  A prefill
step appends q_len new tokens to a sequence whose cache then holds n tokens (the new ones
included, at positions n - q_len .. n - 1); the query at position p attends to the tokens at
positions 0 .. p (causal mask), scores q.k/sqrt(D), softmax over those tokens, weighted sum
of V; query head g uses KV head g // G.  Decode is the special case q_len = 1.

The paged cache is gathered into a contiguous copy first, so block placement cannot matter.
"""
from __future__ import annotations

import math

import numpy as np

from .attention import PoolLayout, attend_contiguous, bf16_bits_to_f64, gather_contiguous


def paged_prefill_attention(pool_bits, lay: PoolLayout, q_bits, q_start, q_len, tables, ctx_len, layer: int,
                            scale: float | None = None, seqs=None):
    """q_bits uint16 [total_q, Hq, D]; sequence s owns rows q_start[s] .. q_start[s] + q_len[s].
    Returns out fp64 [total_q, Hq, D] (rows of sequences not in `seqs` are NaN)."""
    total_q, Hq, D = q_bits.shape
    if scale is None:
        scale = 1.0 / math.sqrt(D)
    out = np.full((total_q, Hq, D), np.nan, dtype=np.float64)
    for s in (range(len(ctx_len)) if seqs is None else seqs):
        n, ql = int(ctx_len[s]), int(q_len[s])
        if ql < 1 or n < ql:
            raise ValueError("need 1 <= q_len <= context length")
        Kb, Vb = gather_contiguous(pool_bits, lay, tables[s], n, layer)
        K, V = bf16_bits_to_f64(Kb), bf16_bits_to_f64(Vb)
        for i in range(ql):
            pos = n - ql + i
            row = int(q_start[s]) + i
            out[row] = attend_contiguous(bf16_bits_to_f64(q_bits[row]), K[:pos + 1], V[:pos + 1], scale)
    return out
