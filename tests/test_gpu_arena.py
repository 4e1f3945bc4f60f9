"""Handle-backed pool memory: a handed-over range is unmapped (its physical memory goes back to the
driver), the offline job keeps computing the same bits, and the range comes back mapped."""
import numpy as np
import pytest
import torch

import synth
from oracle import reclaim as R

pytestmark = pytest.mark.gpu


def test_handed_over_range_is_unmapped_and_comes_back():
    import paper_2604_07874_amd as vkv
    wl = synth.workload("llama8b_small")
    g = wl.geom
    seed = 21
    st = synth.build_state(wl, seed, materialize_pool=False)
    handle_bytes = g.blocks_per_handle * g.block_bytes
    n_handles = g.num_blocks // g.blocks_per_handle
    arena, span = vkv.kv_arena_create(0, handle_bytes, n_handles)
    pool = None
    try:
        pool_t = torch.as_tensor(span, device="cuda:0")          # aliases the arena, no copy
        assert pool_t.data_ptr() == span.address and pool_t.numel() == g.pool_elems and pool_t.dtype == torch.int16
        synth.fill_pool_torch(pool_t, g, seed)
        synth.poison_unused_slots(st, pool_t)
        blocks = pool_t.view(g.num_blocks, g.block_elems)
        tables_t = torch.from_numpy(st.tables).cuda()
        remap_t = torch.empty(g.num_blocks, dtype=torch.int32, device="cuda:0")
        pool = vkv.kv_pool_init(g.num_layers, g.num_q_heads, g.num_kv_heads, g.head_dim, g.num_blocks,
                                g.blocks_per_handle, base=pool_t)
        vkv.kv_pool_attach_arena(pool, arena)
        vkv.kv_pool_adopt(pool, np.flatnonzero(st.live).astype(np.int32))
        info = vkv.kv_attn_plan(pool, st.ctx_len, 1 << 20, wl.chunk_tokens)
        ws = torch.empty(info.workspace_bytes, dtype=torch.uint8, device="cuda:0")
        vkv.kv_attn_bind(pool, ws)
        qs = [torch.from_numpy(synth.query_bits(wl, seed, l).view(np.int16)).cuda() for l in range(g.num_layers)]

        def decode():
            out = torch.full((g.num_layers, wl.num_seqs, g.num_q_heads, g.head_dim), float("nan"), dtype=torch.float32,
                             device="cuda:0")
            for l in range(g.num_layers):
                s_, cur = vkv.kv_attn_run_layer(pool, l, 0, qs[l], tables_t, ws, out[l])
                assert s_ == vkv.VKV_OK
            vkv.kv_attn_check(pool, ws)
            return out.cpu().numpy()

        before = decode()
        assert np.isfinite(before).all()
        lo, hi = wl.reclaim_range
        range_bytes = (hi - lo) * g.block_bytes
        mapped, nbytes = vkv.kv_arena_state(arena, n_handles)
        assert mapped.all() and nbytes == g.pool_bytes
        # nothing may be unmapped that the pool has not handed over
        with pytest.raises(vkv.VkvError) as ei:
            vkv.kv_arena_release(arena, pool, lo, hi)
        assert ei.value.code == vkv.VKV_E_STATE
        stats = vkv.kv_reclaim_range(pool, lo, hi, tables_t, remap_t)
        assert stats.blocks_moved > 0
        orc = R.ReclaimOracle(g.num_blocks, g.blocks_per_handle, st.live, st.tables, None)
        assert orc.reclaim(lo, hi)[0] == R.OK
        assert np.array_equal(tables_t.cpu().numpy(), orc.tables)
        vkv.kv_pool_check_tables(pool, orc.tables)               # no entry points into the range
        torch.cuda.synchronize()
        free0 = torch.cuda.mem_get_info()[0]
        print(f"releasing [{lo},{hi}) = {range_bytes >> 20} MiB", flush=True)
        vkv.kv_arena_release(arena, pool, lo, hi)
        free1 = torch.cuda.mem_get_info()[0]
        assert abs((free1 - free0) - range_bytes) <= (8 << 20), (free0, free1, range_bytes)
        mapped, nbytes = vkv.kv_arena_state(arena, n_handles)
        bph = g.blocks_per_handle
        assert not mapped[lo // bph:hi // bph].any() and mapped[:lo // bph].all() and nbytes == g.pool_bytes - range_bytes
        with pytest.raises(vkv.VkvError) as ei:
            vkv.kv_arena_release(arena, pool, lo, hi)             # twice
        assert ei.value.code == vkv.VKV_E_STATE
        with pytest.raises(vkv.VkvError) as ei:
            vkv.kv_pool_return_range(pool, lo, hi)                # not while it has no memory behind it
        assert ei.value.code == vkv.VKV_E_STATE
        # the offline job goes on, on memory that is all still mapped, with the same bits
        print("decode with the range unmapped", flush=True)
        assert np.array_equal(decode(), before)
        ids = vkv.kv_pool_alloc(pool, 4)
        assert (ids < lo).all()                                   # the allocator stays out of the range
        vkv.kv_pool_free(pool, ids)
        # the online tenant gives the range back: fresh memory at the same addresses
        vkv.kv_arena_restore(arena, pool, lo, hi)
        with pytest.raises(vkv.VkvError) as ei:
            vkv.kv_arena_restore(arena, pool, lo, hi)
        assert ei.value.code == vkv.VKV_E_STATE
        vkv.kv_pool_return_range(pool, lo, hi)
        free2 = torch.cuda.mem_get_info()[0]
        assert abs((free0 - free2)) <= (8 << 20)
        mapped, nbytes = vkv.kv_arena_state(arena, n_handles)
        assert mapped.all() and nbytes == g.pool_bytes
        top = torch.tensor([lo, hi - 1], device="cuda:0")
        blocks[top] = 1234
        torch.cuda.synchronize()
        assert int(blocks[hi - 1, -1]) == 1234 and int(blocks[lo, 0]) == 1234
        assert np.array_equal(decode(), before)
    finally:
        if pool is not None:
            vkv.kv_pool_destroy(pool)
        vkv.kv_arena_destroy(arena)
