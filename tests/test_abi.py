"""The C-ABI library loads without a GPU and exports every symbol the header declares;
host-only entry points (pool bookkeeping, plans) agree with the oracle."""
import os
import re

import numpy as np
import pytest

import synth
from oracle import reclaim as R
from oracle.plan import attention_plan

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def vkv():
    import paper_2604_07874_amd as v
    if not os.path.exists(v.library_path()):
        from paper_2604_07874_amd import build
        build.build(verbose=False)
    return v


def declared_functions():
    text = open(os.path.join(ROOT, "include", "valvekv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:kv|vkv|paged|block)_\w+)\s*\(", text)))


def test_every_declared_symbol_is_exported(vkv):
    names = declared_functions()
    assert {"kv_pool_init", "paged_decode_attn_slice", "kv_reclaim_range", "block_table_rewrite"} <= set(names)
    for n in names:
        assert hasattr(vkv.lib, n), n


def test_binding_mirrors_the_header(vkv):
    for n in declared_functions():
        if n == "vkv_last_error":
            continue
        assert n in vkv.__all__, n


def make_pool(vkv, wl, st):
    g = wl.geom
    p = vkv.kv_pool_init(g.num_layers, g.num_q_heads, g.num_kv_heads, g.head_dim, g.num_blocks, g.blocks_per_handle)
    vkv.kv_pool_adopt(p, np.flatnonzero(st.live).astype(np.int32))
    return p


def test_pool_init_rejects_bad_geometry(vkv):
    for args in [(1, 8, 3, 64, 256, 8), (1, 8, 8, 80, 256, 8), (1, 8, 8, 64, 250, 8), (0, 8, 8, 64, 256, 8),
                 (1, 34, 1, 64, 256, 8)]:
        with pytest.raises(vkv.VkvError) as ei:
            vkv.kv_pool_init(*args)
        assert ei.value.code == vkv.VKV_E_INVAL


def test_allocate_release_interface(vkv):
    p = vkv.kv_pool_init(1, 8, 8, 64, 64, 8)
    assert vkv.kv_pool_alloc(p, 3).tolist() == [0, 1, 2]
    vkv.kv_pool_adopt(p, [5, 7])
    assert vkv.kv_pool_alloc(p, 4).tolist() == [3, 4, 6, 8]
    vkv.kv_pool_free(p, [1, 4])
    assert vkv.kv_pool_alloc(p, 2).tolist() == [1, 4]
    for bad in ([1], [64], [-1], [9, 9]):
        with pytest.raises(vkv.VkvError):
            vkv.kv_pool_adopt(p, bad)
    with pytest.raises(vkv.VkvError):
        vkv.kv_pool_free(p, [10])
    with pytest.raises(vkv.VkvError) as ei:
        vkv.kv_pool_alloc(p, 100)
    assert ei.value.code == vkv.VKV_E_NOSPACE
    live, ranges = vkv.kv_pool_state(p, 64)
    assert np.flatnonzero(live).tolist() == [0, 1, 2, 3, 4, 5, 6, 7, 8] and ranges == []
    vkv.kv_pool_check_tables(p, np.array([[0, 5, -1]], dtype=np.int32))
    with pytest.raises(vkv.VkvError) as ei:
        vkv.kv_pool_check_tables(p, np.array([[0, 9, -1]], dtype=np.int32))
    assert ei.value.code == vkv.VKV_E_STATE
    vkv.kv_pool_destroy(p)


@pytest.mark.parametrize("name", ["tiny", "llama8b", "llama70b_tp8", "offline_batch_small"])
def test_attention_plan_matches_oracle(vkv, name):
    wl = synth.workload(name)
    st = synth.build_state(wl, seed=3, materialize_pool=False)
    g = wl.geom
    p = make_pool(vkv, wl, st)
    for chunk, sb in [(wl.chunk_tokens, wl.slice_bytes), (128, 1 << 22), (2048, 1)]:
        info = vkv.kv_attn_plan(p, st.ctx_len, sb, chunk)
        work, starts = vkv.kv_attn_plan_read(p, info)
        owork, ostarts = attention_plan(st.ctx_len, g.num_kv_heads, g.head_dim, g.block_tokens, chunk, sb)
        assert np.array_equal(work, owork) and np.array_equal(starts, ostarts)
        assert info.kv_bytes_per_layer == int(st.ctx_len.astype(np.int64).sum()) * g.kv_bytes_per_token_layer
        nbytes = owork[:, 3].astype(np.int64) * (4 * g.head_dim)
        assert info.max_slice_kv_bytes == max(int(nbytes[a:b].sum()) for a, b in zip(ostarts[:-1], ostarts[1:]))
    for bad_chunk in (0, 16, 48, 4096):
        with pytest.raises(vkv.VkvError):
            vkv.kv_attn_plan(p, st.ctx_len, 1 << 20, bad_chunk)
    with pytest.raises(vkv.VkvError):
        vkv.kv_attn_plan(p, np.array([5, -1], dtype=np.int32), 1 << 20, 64)
    # a sequence that has left the batch (length 0) gets no work
    ctx0 = st.ctx_len.copy()
    ctx0[0] = 0
    info = vkv.kv_attn_plan(p, ctx0, 1 << 22, 128)
    work, starts = vkv.kv_attn_plan_read(p, info)
    owork, ostarts = attention_plan(ctx0, g.num_kv_heads, g.head_dim, g.block_tokens, 128, 1 << 22)
    assert np.array_equal(work, owork) and np.array_equal(starts, ostarts) and 0 not in work[:, 0]
    info = vkv.kv_attn_plan(p, np.zeros(3, dtype=np.int32), 1 << 22, 128)
    assert info.n_items == 0 and info.n_slices == 0
    vkv.kv_pool_destroy(p)


@pytest.mark.parametrize("name,seed", [("tiny", 0), ("llama8b", 1), ("llama70b_tp8", 2), ("stress_small", 3)])
def test_relocation_plan_matches_oracle(vkv, name, seed):
    wl = synth.workload(name)
    st = synth.build_state(wl, seed=seed, materialize_pool=False)
    g = wl.geom
    p = make_pool(vkv, wl, st)
    orc = R.ReclaimOracle(g.num_blocks, g.blocks_per_handle, st.live, st.tables, None)
    lo, hi = wl.reclaim_range
    remap, stats = vkv.kv_reclaim_plan(p, lo, hi, g.num_blocks)
    status, src, dst, oremap = orc.reclaim(lo, hi)
    assert status == R.OK and np.array_equal(remap, oremap)
    assert stats.blocks_moved == len(src) and stats.bytes_moved == len(src) * g.block_bytes
    # the dry run changed nothing
    live, ranges = vkv.kv_pool_state(p, g.num_blocks)
    assert np.array_equal(live, st.live) and ranges == []
    for lo_, hi_, code in [(lo + 1, hi, vkv.VKV_E_INVAL), (hi, hi, vkv.VKV_E_INVAL), (0, g.num_blocks, vkv.VKV_E_NOSPACE)]:
        with pytest.raises(vkv.VkvError) as ei:
            vkv.kv_reclaim_plan(p, lo_, hi_, g.num_blocks)
        assert ei.value.code == code
    vkv.kv_pool_destroy(p)


def test_device_entry_points_refuse_a_host_only_pool(vkv):
    p = vkv.kv_pool_init(1, 8, 8, 64, 64, 8)
    st = vkv.lib.kv_reclaim_range(p, 56, 64, None, 0, 0, 0, None, None, None, 0, None)
    assert st == vkv.VKV_E_INVAL
    st = vkv.lib.paged_decode_attn_slice(p, 0, 0, None, None, 0, None, None, 0.0, None)
    assert st == vkv.VKV_E_STATE       # no plan yet
    vkv.kv_pool_destroy(p)


def test_prefill_plan_refuses_head_dim_64(vkv):
    p = vkv.kv_pool_init(2, 8, 2, 64, 64, 8)
    try:
        with pytest.raises(vkv.VkvError) as e:
            vkv.kv_prefill_plan(p, np.array([40], dtype=np.int32), np.array([8], dtype=np.int32), 1 << 20, 256)
        assert e.value.code == vkv.VKV_E_INVAL and "head_dim 128" in str(e.value)
    finally:
        vkv.kv_pool_destroy(p)


def test_prefill_merge_is_cut_into_bounded_steps(vkv):
    """Host only: the merge of split tiles is planned as steps whose size follows slice_bytes, one
    step when nothing is split."""
    wl = synth.workload("llama8b_small")
    st = synth.build_state(wl, 5, materialize_pool=False)
    p = make_pool(vkv, wl, st)
    try:
        q_len = np.minimum(st.ctx_len, 4096).astype(np.int32)
        whole = vkv.kv_prefill_plan(p, st.ctx_len, q_len, 1 << 40, 16384)     # every tile is one chunk
        assert whole.n_merge_steps == 1 and whole.n_slices == 1
        coarse = vkv.kv_prefill_plan(p, st.ctx_len, q_len, 64 << 20, 256)
        fine = vkv.kv_prefill_plan(p, st.ctx_len, q_len, 1 << 20, 256)
        assert 1 <= coarse.n_merge_steps < fine.n_merge_steps
        assert fine.n_items == coarse.n_items and fine.n_slices > coarse.n_slices
    finally:
        vkv.kv_pool_destroy(p)
