"""Pins for the causal prefill oracle."""
import math

import numpy as np
import pytest
import torch

import synth
from oracle.attention import PoolLayout, bf16_bits_to_f64, gather_contiguous, paged_decode_attention
from oracle.prefill import paged_prefill_attention


def case(seed=0, q_lens=(5, 40, 17)):
    wl = synth.workload("llama8b_small", geom=synth.Geometry(2, 8, 2, 64, 96, 8), num_seqs=3,
                        ctx_dist=("uniform", 41, 150), occupancy=0.6)
    st = synth.build_state(wl, seed=seed)
    g = wl.geom
    lay = PoolLayout(g.num_layers, g.num_kv_heads, g.head_dim, g.block_tokens)
    q_len = np.minimum(np.asarray(q_lens), st.ctx_len).astype(np.int32)
    q_start = np.concatenate([[0], np.cumsum(q_len)[:-1]]).astype(np.int32)
    total = int(q_len.sum())
    q = synth.hash_bf16_bits(np.arange(total * g.num_q_heads * g.head_dim, dtype=np.int64), seed, 1)
    return wl, st, lay, q.reshape(total, g.num_q_heads, g.head_dim), q_start, q_len


def test_matches_library_sdpa_with_causal_mask():
    wl, st, lay, q, q_start, q_len = case()
    g = wl.geom
    out = paged_prefill_attention(st.pool_bits, lay, q, q_start, q_len, st.tables, st.ctx_len, 1)
    assert np.isfinite(out).all()
    for s in range(3):
        n, ql = int(st.ctx_len[s]), int(q_len[s])
        Kb, Vb = gather_contiguous(st.pool_bits, lay, st.tables[s], n, 1)
        K = torch.from_numpy(bf16_bits_to_f64(Kb)).permute(1, 0, 2).repeat_interleave(g.group, dim=0)   # [Hq, n, D]
        V = torch.from_numpy(bf16_bits_to_f64(Vb)).permute(1, 0, 2).repeat_interleave(g.group, dim=0)
        Q = torch.from_numpy(bf16_bits_to_f64(q[q_start[s]:q_start[s] + ql])).permute(1, 0, 2)           # [Hq, ql, D]
        # query i sits at position n - ql + i and sees tokens 0 .. n - ql + i
        mask = torch.arange(n)[None, :] <= (n - ql + torch.arange(ql))[:, None]
        ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V, attn_mask=mask).permute(1, 0, 2).numpy()
        assert np.max(np.abs(out[q_start[s]:q_start[s] + ql] - ref)) <= 1e-12


def test_last_query_equals_decode_and_first_query_of_a_full_prefill_sees_one_token():
    wl, st, lay, q, q_start, q_len = case(seed=2)
    out = paged_prefill_attention(st.pool_bits, lay, q, q_start, q_len, st.tables, st.ctx_len, 0)
    last = q[q_start + q_len - 1]                                  # [S, Hq, D]
    dec = paged_decode_attention(st.pool_bits, lay, last, st.tables, st.ctx_len, 0)
    assert np.array_equal(out[q_start + q_len - 1], dec)
    # whole sequence as one prefill: the query at position 0 returns V[0] exactly
    full = st.ctx_len.copy()
    qs = np.concatenate([[0], np.cumsum(full)[:-1]]).astype(np.int32)
    g = wl.geom
    qq = synth.hash_bf16_bits(np.arange(int(full.sum()) * g.num_q_heads * g.head_dim, dtype=np.int64), 9, 1)
    qq = qq.reshape(int(full.sum()), g.num_q_heads, g.head_dim)
    out2 = paged_prefill_attention(st.pool_bits, lay, qq, qs, full, st.tables, st.ctx_len, 0, seqs=[1])
    _, Vb = gather_contiguous(st.pool_bits, lay, st.tables[1], 1, 0)
    for h in range(g.num_q_heads):
        assert np.array_equal(out2[qs[1], h], bf16_bits_to_f64(Vb[0, h // g.group]))


def test_future_tokens_do_not_matter():
    # changing K/V of a token changes only the outputs of queries at or after its position
    wl, st, lay, q, q_start, q_len = case(seed=3)
    s = 1
    n, ql = int(st.ctx_len[s]), int(q_len[s])
    out0 = paged_prefill_attention(st.pool_bits, lay, q, q_start, q_len, st.tables, st.ctx_len, 0, seqs=[s])
    pool2 = st.pool_bits.copy()
    t = n - ql + ql // 2                                   # a token in the middle of the new chunk
    blk = int(st.tables[s, t // 16])
    for kv in (0, 1):
        for h in range(wl.geom.num_kv_heads):
            o = lay.vec_offset(blk, 0, kv, h, t % 16)
            pool2[o:o + wl.geom.head_dim] ^= 0x0100        # flip a mantissa bit
    out1 = paged_prefill_attention(pool2, lay, q, q_start, q_len, st.tables, st.ctx_len, 0, seqs=[s])
    rows = np.arange(q_start[s], q_start[s] + ql)
    changed = np.any(out0[rows] != out1[rows], axis=(1, 2))
    assert not changed[:ql // 2].any() and changed[ql // 2:].all()


def test_rejects_bad_lengths():
    wl, st, lay, q, q_start, q_len = case()
    bad = q_len.copy()
    bad[0] = 0
    with pytest.raises(ValueError):
        paged_prefill_attention(st.pool_bits, lay, q, q_start, bad, st.tables, st.ctx_len, 0)
    bad[0] = int(st.ctx_len[0]) + 1
    with pytest.raises(ValueError):
        paged_prefill_attention(st.pool_bits, lay, q, q_start, bad, st.tables, st.ctx_len, 0)
