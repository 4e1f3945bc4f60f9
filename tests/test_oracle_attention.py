"""Pins for the fp64 attention oracle: things the mathematics fixes, none derived from the oracle."""
import math
import struct

import numpy as np
import pytest
import torch

import synth
from oracle.attention import (PoolLayout, bf16_bits_to_f64, gather_contiguous,
                              paged_decode_attention)


def layout_of(g):
    return PoolLayout(g.num_layers, g.num_kv_heads, g.head_dim, g.block_tokens)


def f32_to_bf16_bits(x):
    u = np.asarray(x, dtype=np.float32).view(np.uint32)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def bits_val(b):
    return struct.unpack("<f", struct.pack("<I", int(b) << 16))[0]


@pytest.fixture(scope="module")
def tiny():
    wl = synth.workload("tiny")
    st = synth.build_state(wl, seed=0)
    return wl, st, synth.query_bits(wl, 0, 0)


# ---------------------------------------------------------------- brute force
def scalar_attention(pool, L, Hkv, D, B, q_bits, tables, ctx, layer):
    """Pure-Python scalar loops with their own address arithmetic."""
    S, Hq = len(q_bits), len(q_bits[0])
    G = Hq // Hkv
    out = np.zeros((S, Hq, D))
    for s in range(S):
        n = int(ctx[s])
        for g in range(Hq):
            h = g // G
            qv = [bits_val(q_bits[s][g][d]) for d in range(D)]
            xs = []
            for t in range(n):
                blk = int(tables[s][t // B])
                base = blk * (L * 2 * Hkv * B * D) + layer * (2 * Hkv * B * D) \
                    + 0 * (Hkv * B * D) + h * (B * D) + (t % B) * D
                xs.append(sum(qv[d] * bits_val(pool[base + d]) for d in range(D)) / math.sqrt(D))
            m = max(xs)
            es = [math.exp(x - m) for x in xs]
            z = math.fsum(es)
            for t in range(n):
                blk = int(tables[s][t // B])
                base = blk * (L * 2 * Hkv * B * D) + layer * (2 * Hkv * B * D) \
                    + 1 * (Hkv * B * D) + h * (B * D) + (t % B) * D
                w = es[t] / z
                for d in range(D):
                    out[s, g, d] += w * bits_val(pool[base + d])
    return out


def test_matches_scalar_brute_force(tiny):
    wl, st, q = tiny
    g = wl.geom
    ref = scalar_attention(st.pool_bits, g.num_layers, g.num_kv_heads, g.head_dim, g.block_tokens,
                           q, st.tables, st.ctx_len, 0)
    out = paged_decode_attention(st.pool_bits, layout_of(g), q, st.tables, st.ctx_len, 0)
    assert np.max(np.abs(out - ref)) <= 1e-12


def test_matches_library_sdpa_on_contiguous_copy():
    wl = synth.workload("llama8b_small", geom=synth.Geometry(2, 8, 2, 128, 64, 8), num_seqs=3,
                        ctx_dist=("uniform", 5, 200), occupancy=0.6)
    st = synth.build_state(wl, seed=3)
    g = wl.geom
    lay = layout_of(g)
    for layer in (0, 1):
        q = synth.query_bits(wl, 3, layer)
        out = paged_decode_attention(st.pool_bits, lay, q, st.tables, st.ctx_len, layer)
        for s in range(wl.num_seqs):
            Kb, Vb = gather_contiguous(st.pool_bits, lay, st.tables[s], int(st.ctx_len[s]), layer)
            K = torch.from_numpy(bf16_bits_to_f64(Kb)).permute(1, 0, 2)   # [Hkv, n, D]
            V = torch.from_numpy(bf16_bits_to_f64(Vb)).permute(1, 0, 2)
            K = K.repeat_interleave(g.group, dim=0)                        # query head g -> kv head g // G
            V = V.repeat_interleave(g.group, dim=0)
            Q = torch.from_numpy(bf16_bits_to_f64(q[s])).unsqueeze(1)      # [Hq, 1, D]
            ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V).squeeze(1).numpy()
            assert np.max(np.abs(out[s] - ref)) <= 1e-12


# ---------------------------------------------------------------- closed forms
def small_case(L=2, Hq=4, Hkv=2, D=8, NB=12, n=(1, 23, 37), seed=11):
    """Hand-built pool: random bf16 values, tables chosen by a seeded shuffle."""
    rng = np.random.default_rng(seed)
    lay = PoolLayout(L, Hkv, D, 16)
    pool = f32_to_bf16_bits(rng.standard_normal(NB * lay.block_elems))
    ctx = np.asarray(n, dtype=np.int32)
    ids = list(rng.permutation(NB))
    tables = np.full((len(n), 4), -1, dtype=np.int32)
    for s, ns in enumerate(n):
        for j in range(-(-ns // 16)):
            tables[s, j] = ids.pop()
    q = f32_to_bf16_bits(rng.standard_normal((len(n), Hq, D)))
    return lay, pool, q, tables, ctx


def set_vec(pool, lay, blk, layer, kv, h, slot, values):
    o = lay.vec_offset(blk, layer, kv, h, slot)
    pool[o:o + lay.head_dim] = f32_to_bf16_bits(values)


def test_single_token_returns_its_value_row():
    lay, pool, q, tables, ctx = small_case()
    out = paged_decode_attention(pool, lay, q, tables, ctx, 1)
    for g in range(4):
        o = lay.vec_offset(int(tables[0, 0]), 1, 1, g // 2, 0)
        assert np.array_equal(out[0, g], bf16_bits_to_f64(pool[o:o + 8]))


def test_zero_query_gives_mean_of_values():
    lay, pool, q, tables, ctx = small_case()
    q[:] = 0
    out = paged_decode_attention(pool, lay, q, tables, ctx, 0)
    for s in range(3):
        _, Vb = gather_contiguous(pool, lay, tables[s], int(ctx[s]), 0)
        V = bf16_bits_to_f64(Vb)
        for g in range(4):
            assert np.allclose(out[s, g], V[:, g // 2].mean(axis=0), rtol=0, atol=1e-14)


def test_constant_value_per_kv_head_pins_gqa_mapping_and_kv_index():
    # V of kv head h in layer l is the constant 1 + h + 10*l; K is left random.
    lay, pool, q, tables, ctx = small_case()
    for blk in range(12):
        for layer in range(2):
            for h in range(2):
                for slot in range(16):
                    set_vec(pool, lay, blk, layer, 1, h, slot, np.full(8, 1.0 + h + 10 * layer))
    for layer in range(2):
        out = paged_decode_attention(pool, lay, q, tables, ctx, layer)
        for g in range(4):
            assert np.allclose(out[:, g], 1.0 + (g // 2) + 10 * layer, rtol=0, atol=1e-13)


@pytest.mark.parametrize("tstar", [0, 15, 16, 22, 36])
def test_dominant_key_selects_its_token(tstar):
    # Token t* gets a key aligned with q (huge score); its V row is a marker.
    lay, pool, q, tables, ctx = small_case()
    s, layer, D = 2, 1, 8
    qv = bf16_bits_to_f64(q[s])
    for h in range(2):
        g = 2 * h  # first query head of the group
        blk, slot = int(tables[s, tstar // 16]), tstar % 16
        set_vec(pool, lay, blk, layer, 0, h, slot, 64.0 * qv[g] / max(1e-3, np.dot(qv[g], qv[g])) * 8)
        set_vec(pool, lay, blk, layer, 1, h, slot, np.arange(D) + 100.0 * (h + 1))
    out = paged_decode_attention(pool, lay, q, tables, ctx, layer)
    for h in range(2):
        # score of t* is about 512/sqrt(8) = 181 above the rest (|other scores| < 20)
        assert np.allclose(out[s, 2 * h], np.arange(D) + 100.0 * (h + 1), rtol=0, atol=1e-9)


# ---------------------------------------------------------------- invariants
def test_output_in_convex_hull_of_values(tiny):
    wl, st, q = tiny
    lay = layout_of(wl.geom)
    out = paged_decode_attention(st.pool_bits, lay, q, st.tables, st.ctx_len, 0)
    for s in range(wl.num_seqs):
        _, Vb = gather_contiguous(st.pool_bits, lay, st.tables[s], int(st.ctx_len[s]), 0)
        V = bf16_bits_to_f64(Vb)
        for g in range(wl.geom.num_q_heads):
            h = g // wl.geom.group
            assert np.all(out[s, g] <= V[:, h].max(axis=0) + 1e-12)
            assert np.all(out[s, g] >= V[:, h].min(axis=0) - 1e-12)


def test_paged_equals_contiguous_under_block_relabelling(tiny):
    # Moving every block to another physical id (and renaming table entries) changes nothing.
    wl, st, q = tiny
    g = wl.geom
    lay = layout_of(g)
    out0 = paged_decode_attention(st.pool_bits, lay, q, st.tables, st.ctx_len, 0)
    perm = np.random.default_rng(1).permutation(g.num_blocks)
    pool2 = np.empty_like(st.pool_bits).reshape(g.num_blocks, -1)
    pool2[perm] = st.pool_bits.reshape(g.num_blocks, -1)
    tables2 = np.where(st.tables >= 0, perm[np.maximum(st.tables, 0)], -1).astype(np.int32)
    out1 = paged_decode_attention(pool2.reshape(-1), lay, q, tables2, st.ctx_len, 0)
    assert np.array_equal(out0, out1)


def test_token_permutation_invariance():
    lay, pool, q, tables, ctx = small_case(n=(32, 48, 16))
    out0 = paged_decode_attention(pool, lay, q, tables, ctx, 0)
    t2 = tables.copy()
    t2[1, :3] = tables[1, [2, 0, 1]]  # whole blocks of 16 tokens reordered
    out1 = paged_decode_attention(pool, lay, q, t2, ctx, 0)
    assert np.allclose(out0, out1, rtol=0, atol=1e-13)


def test_unused_slots_are_never_read(tiny):
    wl, st, q = tiny
    assert st.poisoned, "the tiny workload must have ragged last blocks"
    out = paged_decode_attention(st.pool_bits, layout_of(wl.geom), q, st.tables, st.ctx_len, 0)
    assert np.isfinite(out).all()


def test_rejects_empty_context_and_missing_blocks():
    lay, pool, q, tables, ctx = small_case()
    bad = ctx.copy()
    bad[1] = 0
    with pytest.raises(ValueError):
        paged_decode_attention(pool, lay, q, tables, bad, 0)
    t2 = tables.copy()
    t2[2, 1] = -1
    with pytest.raises(ValueError):
        paged_decode_attention(pool, lay, q, t2, ctx, 0)


def test_softmax_shift_invariance():
    # Adding c*q/|q|^2 to every key adds the same constant to every score of that head.
    from oracle.attention import attend_contiguous
    rng = np.random.default_rng(5)
    q = rng.standard_normal((4, 16))
    K = rng.standard_normal((50, 1, 16))
    V = rng.standard_normal((50, 1, 16))
    out0 = attend_contiguous(q[:1], K, V, 0.25)
    K2 = K + 3.0 * q[0] / np.dot(q[0], q[0])
    out1 = attend_contiguous(q[:1], K2, V, 0.25)
    assert np.allclose(out0, out1, rtol=0, atol=1e-12)
