"""fp64 decode attention over a paged bf16 KV cache (test oracle).

Definition followed: one decode query per sequence attends over all of that
sequence's cached tokens (the new token's K/V already appended); scores are
q.k/sqrt(D), weights their softmax over tokens, output the weighted sum of V.
Query head g reads KV head g // G (grouped-query attention).  The paged cache
is first gathered into a contiguous [tokens, kv_heads, D] copy through the
block table, so the result cannot depend on where blocks sit in the pool: this
is the property the paper's reclamation must preserve for the offline job to
"resume later" (Section 5, "Sub-layer memory reclamation").

All arithmetic is fp64 on the exact values of the bf16 bit patterns.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class PoolLayout:
    """pool[block][layer][K|V][kv_head][slot][d], bf16 elements."""
    num_layers: int
    num_kv_heads: int
    head_dim: int
    block_tokens: int = 16

    @property
    def block_elems(self) -> int:
        return self.num_layers * 2 * self.num_kv_heads * self.block_tokens * self.head_dim

    def vec_offset(self, block: int, layer: int, kv: int, head: int, slot: int) -> int:
        return ((((block * self.num_layers + layer) * 2 + kv) * self.num_kv_heads + head)
                * self.block_tokens + slot) * self.head_dim


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to fp64."""
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def gather_contiguous(pool_bits: np.ndarray, lay: PoolLayout, table_row: np.ndarray,
                      n_tokens: int, layer: int):
    """Contiguous K, V copies, each uint16 [n_tokens, kv_heads, D], of one sequence."""
    H, D, B = lay.num_kv_heads, lay.head_dim, lay.block_tokens
    K = np.empty((n_tokens, H, D), dtype=np.uint16)
    V = np.empty((n_tokens, H, D), dtype=np.uint16)
    for t in range(n_tokens):
        blk = int(table_row[t // B])
        if blk < 0:
            raise ValueError(f"token {t} maps to an empty table entry")
        slot = t % B
        for h in range(H):
            o = lay.vec_offset(blk, layer, 0, h, slot)
            K[t, h] = pool_bits[o:o + D]
            o = lay.vec_offset(blk, layer, 1, h, slot)
            V[t, h] = pool_bits[o:o + D]
    return K, V


def attend_contiguous(q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float) -> np.ndarray:
    """q [Hq, D], K/V [n, Hkv, D], all fp64 -> out [Hq, D] fp64."""
    Hq, D = q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    out = np.empty((Hq, D), dtype=np.float64)
    for g in range(Hq):
        h = g // G
        x = (K[:, h, :] @ q[g]) * scale
        x = x - x.max()
        p = np.exp(x)
        p = p / p.sum()
        out[g] = p @ V[:, h, :]
    return out


def paged_decode_attention(pool_bits: np.ndarray, lay: PoolLayout, q_bits: np.ndarray,
                           tables: np.ndarray, ctx_len: np.ndarray, layer: int,
                           scale: float | None = None, seqs=None) -> np.ndarray:
    """out fp64 [S, Hq, D] (rows of sequences not in `seqs` are left NaN)."""
    S, Hq, D = q_bits.shape
    assert D == lay.head_dim and Hq % lay.num_kv_heads == 0
    if scale is None:
        scale = 1.0 / math.sqrt(D)
    out = np.full((S, Hq, D), np.nan, dtype=np.float64)
    for s in (range(S) if seqs is None else seqs):
        n = int(ctx_len[s])
        if n < 1:
            raise ValueError("context length must be at least 1")
        Kb, Vb = gather_contiguous(pool_bits, lay, tables[s], n, layer)
        out[s] = attend_contiguous(bf16_bits_to_f64(q_bits[s]), bf16_bits_to_f64(Kb),
                                   bf16_bits_to_f64(Vb), scale)
    return out
