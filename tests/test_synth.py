"""The seeded input generator: host and torch paths agree; states are well formed."""
import numpy as np
import pytest
import torch

import synth


def test_hash_numpy_equals_torch():
    idx = np.concatenate([np.arange(4096, dtype=np.int64),
                          np.arange(4096, dtype=np.int64) + (1 << 37) + 12345])
    for seed, stream in [(0, 0), (7, 1), (123456789, 0)]:
        a = synth.hash_bf16_bits(idx, seed, stream)
        b = synth.hash_bf16_bits_torch(torch.from_numpy(idx), seed, stream).numpy().view(np.uint16)
        assert np.array_equal(a, b)


def test_hash_distribution_is_standard_normal_like():
    a = synth.hash_bf16_bits(np.arange(1 << 18, dtype=np.int64), 1, 0)
    x = (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert abs(x.mean()) < 0.01 and abs(x.std() - 1.0) < 0.01
    assert np.isfinite(x).all() and np.abs(x).max() < 5.0
    assert abs(np.mean(np.abs(x) < 1.0) - 0.6827) < 0.01


def test_fill_pool_torch_matches_block_regeneration():
    wl = synth.workload("tiny")
    g = wl.geom
    pool = torch.empty(g.pool_elems, dtype=torch.int16)
    synth.fill_pool_torch(pool, g, seed=5, chunk_elems=1 << 20)
    ids = [0, 3, 255]
    ref = synth.pool_bits_for_blocks(g, 5, ids)
    got = pool.numpy().view(np.uint16).reshape(g.num_blocks, g.block_elems)[ids]
    assert np.array_equal(ref, got)


@pytest.mark.parametrize("name", ["tiny", "llama8b", "llama70b_tp8", "llama8b_small",
                                  "offline_batch_small", "llama70b_tp8_small", "stress_small"])
def test_state_is_well_formed(name):
    wl = synth.workload(name)
    st = synth.build_state(wl, seed=2, materialize_pool=False)
    g = wl.geom
    S = wl.num_seqs
    assert st.ctx_len.shape == (S,) and st.ctx_len.min() >= 1 and st.ctx_len.max() <= wl.ctx_cap
    used = st.tables[st.tables >= 0]
    assert len(np.unique(used)) == len(used)           # no sharing unless asked for
    assert st.live.sum() == len(used)                  # every live block is referenced
    assert np.all(st.live[used] == 1)
    for s in range(S):
        nb = -(-int(st.ctx_len[s]) // g.block_tokens)
        assert np.all(st.tables[s, :nb] >= 0) and np.all(st.tables[s, nb:] == -1)
    if wl.occupancy is not None:
        assert st.live.sum() >= round(wl.occupancy * g.num_blocks)
    lo, hi = wl.reclaim_range
    assert lo % g.blocks_per_handle == 0 and hi == g.num_blocks
    # enough room outside the range for what lives inside it
    assert (st.live[:lo] == 0).sum() >= st.live[lo:hi].sum()


def test_shared_prefix_and_poison():
    wl = synth.workload("tiny", shared_prefix_blocks=1, ctx_dist=("uniform", 40, 200))
    st = synth.build_state(wl, seed=4)
    assert st.tables[1, 0] == st.tables[0, 0]
    g = wl.geom
    for blk, used in st.poisoned:
        o = g.elem_offset(blk, 0, 1, 3, used)
        assert np.all(st.pool_bits[o:o + g.head_dim] == synth.BF16_NAN_BITS)
        o = g.elem_offset(blk, 0, 0, 0, used - 1)
        assert np.all(st.pool_bits[o:o + g.head_dim] != synth.BF16_NAN_BITS)


def test_dump_state_round_trip(tmp_path):
    """The flat file the native counter driver reads holds exactly the generator's state."""
    from synth.dump_state import MAGIC, dump
    name, seed = "llama8b_small", 5
    path = tmp_path / "state.bin"
    dump(name, seed, str(path))
    wl = synth.workload(name)
    g = wl.geom
    st = synth.build_state(wl, seed, materialize_pool=False)
    raw = path.read_bytes()
    head = np.frombuffer(raw, dtype="<i4", count=16)
    lo, hi = wl.reclaim_range
    assert head.tolist() == [MAGIC, 1, g.num_layers, g.num_q_heads, g.num_kv_heads, g.head_dim, g.num_blocks,
                             g.blocks_per_handle, wl.num_seqs, st.tables.shape[0], st.tables.shape[1], lo, hi,
                             wl.chunk_tokens, 0, 0]
    off = 64
    sizes = np.frombuffer(raw, dtype="<i8", count=2, offset=off)
    assert sizes.tolist() == [wl.slice_bytes, wl.chunk_bytes]
    off += 16
    ctx = np.frombuffer(raw, dtype="<i4", count=wl.num_seqs, offset=off)
    off += 4 * wl.num_seqs
    tables = np.frombuffer(raw, dtype="<i4", count=st.tables.size, offset=off).reshape(st.tables.shape)
    off += 4 * st.tables.size
    live = np.frombuffer(raw, dtype=np.uint8, count=g.num_blocks, offset=off)
    assert off + g.num_blocks == len(raw)
    assert np.array_equal(ctx, st.ctx_len) and np.array_equal(tables, st.tables) and np.array_equal(live, st.live)
