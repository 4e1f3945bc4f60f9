"""GPU: the eviction fallback in the path.  When a burst's relocation finds no room, handles chosen by
Algorithm 1 are handed over without a copy, the evicted requests' rows are cleared on the device, and
the surviving sequences keep computing the same bits (Section 5, "Sub-layer memory reclamation" and
"Selective handle reclamation")."""
import numpy as np
import pytest
import torch

import synth
from oracle import reclaim as R

pytestmark = pytest.mark.gpu


def costs_of(st, wl):
    """Cost(r) = tokens request r would have to recompute: its context length (background rows: the
    tokens their blocks hold)."""
    n_rows = st.tables.shape[0]
    cost = np.array([int((st.tables[r] >= 0).sum()) * 16 for r in range(n_rows)], dtype=np.int64)
    cost[:wl.num_seqs] = st.ctx_len
    return cost


def test_overlapping_bursts_relocate_then_evict_and_survivors_keep_their_bits():
    from gpu_util import DeviceCase
    wl = synth.workload("stress_small")
    c = DeviceCase(wl, seed=41)
    try:
        vkv, g = c.vkv, wl.geom
        bph, nb, S = g.blocks_per_handle, g.num_blocks, wl.num_seqs
        cost = costs_of(c.st, wl)
        orc = R.ReclaimOracle(nb, bph, c.st.live, c.st.tables, None)
        tables_host = c.st.tables.copy()
        c.plan(slice_bytes=1 << 19, chunk_tokens=128)
        q, q_t = c.q_dev(1)
        clean = c.attention(1, q_t)
        blocks = c.pool_t.view(nb, g.block_elems)

        # first burst: the top two handles; relocation fits
        lo1, hi1 = nb - 2 * bph, nb
        status, mode, payload = orc.reclaim_or_evict(lo1, hi1, cost.tolist())
        assert (status, mode) == (R.OK, 0)
        info, stats, handles, evicted, inv = vkv.kv_reclaim_or_evict(c.pool, lo1, hi1, c.tables_t, tables_host, cost, c.remap_t)
        assert info.mode == 0 and stats.blocks_moved == len(payload[0]) > 0 and len(evicted) == 0
        assert np.array_equal(c.tables_t.cpu().numpy(), orc.tables) and np.array_equal(tables_host, orc.tables)
        assert np.array_equal(c.attention(1, q_t), clean)

        # second burst while the first range is still held: the next two handles; no room any more
        lo2, hi2 = nb - 4 * bph, nb - 2 * bph
        with pytest.raises(vkv.VkvError) as e:
            vkv.kv_reclaim_plan(c.pool, lo2, hi2, nb)
        assert e.value.code == vkv.VKV_E_NOSPACE
        status, mode, payload = orc.reclaim_or_evict(lo2, hi2, cost.tolist())
        assert (status, mode) == (R.OK, 1)
        o_handles, o_evicted, o_inv, o_total = payload
        info, stats, handles, evicted, (rows, cols, blks) = vkv.kv_reclaim_or_evict(
            c.pool, lo2, hi2, c.tables_t, tables_host, cost, c.remap_t)
        assert info.mode == 1 and info.n_handles == 2 and info.total_cost == o_total
        assert handles.tolist() == o_handles and evicted.tolist() == o_evicted
        assert list(zip(rows.tolist(), cols.tolist(), blks.tolist())) == o_inv
        assert len(set(evicted.tolist())) == len(evicted)                   # every evicted request once
        assert np.array_equal(c.tables_t.cpu().numpy(), orc.tables) and np.array_equal(tables_host, orc.tables)
        live, ranges = vkv.kv_pool_state(c.pool, nb)
        assert np.array_equal(live, orc.live) and ranges == orc.released
        vkv.kv_pool_check_tables(c.pool, tables_host)
        print(f"evicted handles {handles.tolist()} at cost {info.total_cost}: rows {evicted.tolist()}, "
              f"{info.n_invalidated} invalidated entries", flush=True)

        # the online tenant scribbles over everything it was handed
        for rlo, rhi in ranges:
            blocks[rlo:rhi] = synth.BF16_NAN_BITS
        # the next decode step: evicted batch sequences have left (context length 0), the others are untouched
        ctx = c.st.ctx_len.copy()
        gone = [r for r in evicted.tolist() if r < S]
        ctx[gone] = 0
        survivors = [s for s in range(S) if s not in gone]
        assert survivors, "the example must leave somebody"
        c.plan(slice_bytes=1 << 19, chunk_tokens=128, ctx=ctx)
        after = c.attention(1, q_t)
        assert np.array_equal(after[survivors], clean[survivors])
        assert np.isnan(after[gone]).all()                                   # nothing was written for the ones that left

        # a third burst finds the evicted requests gone: nobody is reported twice
        status, mode, payload = orc.reclaim_or_evict(nb - 6 * bph, nb - 4 * bph, cost.tolist())
        info3, _, handles3, evicted3, _ = vkv.kv_reclaim_or_evict(c.pool, nb - 6 * bph, nb - 4 * bph, c.tables_t, tables_host,
                                                                  cost, c.remap_t)
        assert status == R.OK and info3.mode == mode
        assert not set(evicted3.tolist()) & set(evicted.tolist())
        assert np.array_equal(c.tables_t.cpu().numpy(), orc.tables) and np.array_equal(tables_host, orc.tables)
        live, ranges = vkv.kv_pool_state(c.pool, nb)
        assert np.array_equal(live, orc.live) and ranges == orc.released
    finally:
        c.close()


def test_invalidate_with_device_tables_and_what_may_be_unmapped():
    """kv_invalidate_handles with the device tables in hand clears the entries there and makes the handles
    safe to unmap; without them the arena refuses.  Slices that meet the cleared entries skip them and
    raise the flag instead of touching unmapped memory."""
    import paper_2604_07874_amd as vkv
    wl = synth.workload("llama8b_small")
    g = wl.geom
    seed = 23
    st = synth.build_state(wl, seed, materialize_pool=False)
    bph = g.blocks_per_handle
    n_handles = g.num_blocks // bph
    arena, span = vkv.kv_arena_create(0, bph * g.block_bytes, n_handles)
    pool = None
    try:
        pool_t = torch.as_tensor(span, device="cuda:0")
        synth.fill_pool_torch(pool_t, g, seed)
        synth.poison_unused_slots(st, pool_t)
        tables_t = torch.from_numpy(st.tables).cuda()
        remap_t = torch.empty(g.num_blocks, dtype=torch.int32, device="cuda:0")
        pool = vkv.kv_pool_init(g.num_layers, g.num_q_heads, g.num_kv_heads, g.head_dim, g.num_blocks, bph, base=pool_t)
        vkv.kv_pool_attach_arena(pool, arena)
        vkv.kv_pool_adopt(pool, np.flatnonzero(st.live).astype(np.int32))
        info = vkv.kv_attn_plan(pool, st.ctx_len, 1 << 20, 256)
        ws = torch.empty(info.workspace_bytes, dtype=torch.uint8, device="cuda:0")
        q_t = torch.from_numpy(synth.query_bits(wl, seed, 0).view(np.int16)).cuda()

        def decode():
            vkv.kv_attn_bind(pool, ws)
            out = torch.full((wl.num_seqs, g.num_q_heads, g.head_dim), float("nan"), dtype=torch.float32, device="cuda:0")
            s_, _ = vkv.kv_attn_run_layer(pool, 0, 0, q_t, tables_t, ws, out)
            assert s_ == vkv.VKV_OK
            return out

        before = decode()
        vkv.kv_attn_check(pool, ws)
        # two handles that batch sequences have blocks in
        used = np.unique(st.tables[:wl.num_seqs][st.tables[:wl.num_seqs] >= 0] // bph)
        h_host, h_dev = int(used[0]), int(used[-1])
        # host tables only: handed over, but not to be unmapped
        vkv.kv_invalidate_handles(pool, [h_host], st.tables)
        with pytest.raises(vkv.VkvError) as e:
            vkv.kv_arena_release(arena, pool, h_host * bph, (h_host + 1) * bph)
        assert e.value.code == vkv.VKV_E_STATE and "device block tables" in str(e.value)
        # with the device tables: entries cleared there, handle unmapped, decode skips and flags
        rows, cols, blks = vkv.kv_invalidate_handles(pool, [h_dev], st.tables, tables_dev=tables_t, remap_dev=remap_t)
        assert len(rows) > 0 and (blks // bph == h_dev).all()
        tabs = tables_t.cpu().numpy()
        assert (tabs[rows, cols] == -1).all()
        keep = np.ones_like(tabs, dtype=bool)
        keep[rows, cols] = False
        assert np.array_equal(tabs[keep], st.tables[keep])
        vkv.kv_arena_release(arena, pool, h_dev * bph, (h_dev + 1) * bph)
        out = decode()                                   # would fault if a cleared entry were still followed
        with pytest.raises(vkv.VkvError) as e:
            vkv.kv_attn_check(pool, ws)
        assert e.value.code == vkv.VKV_E_STATE
        hit = sorted(set(int(r) for r in rows if r < wl.num_seqs) |
                     {s for s in range(wl.num_seqs) if (st.tables[s][st.tables[s] >= 0] // bph == h_host).any()})
        untouched = [s for s in range(wl.num_seqs) if s not in hit]
        assert untouched
        assert torch.equal(out[untouched], before[untouched])
        vkv.kv_arena_restore(arena, pool, h_dev * bph, (h_dev + 1) * bph)
    finally:
        if pool is not None:
            vkv.kv_pool_destroy(pool)
        vkv.kv_arena_destroy(arena)


def test_grace_wait_covers_the_default_stream():
    """Decode on the default stream, reclamation on a side stream, decode_stream passed as the default
    stream (a NULL handle): the call returns only after the slices enqueued before it have finished."""
    from gpu_util import DeviceCase
    wl = synth.workload("offline_batch_small")
    c = DeviceCase(wl, seed=43)
    try:
        vkv, g = c.vkv, wl.geom
        c.plan(slice_bytes=1 << 30, chunk_tokens=2048)
        q, q_t = c.q_dev(0)
        out = torch.empty((wl.num_seqs, g.num_q_heads, g.head_dim), dtype=torch.float32, device="cuda:0")
        default = torch.cuda.default_stream()
        assert default.cuda_stream == 0
        side = torch.cuda.Stream()
        a = torch.randn(8192, 8192, device="cuda:0")
        torch.cuda.synchronize()
        with torch.cuda.stream(default):
            for _ in range(40):                         # tens of milliseconds of other work in the queue first
                a = a @ a * 1e-4
            vkv.paged_decode_attn_slice(c.pool, 0, 0, q_t, c.tables_t, c.ws, out, stream=default)
        marker = torch.cuda.Event()
        marker.record(default)
        assert not marker.query()                       # the slice is still waiting behind that work
        lo, hi = wl.reclaim_range
        vkv.kv_reclaim_range(c.pool, lo, hi, c.tables_t, c.remap_t, copy_stream=side, decode_stream=default)
        assert marker.query()                           # the grace wait saw the default stream's work out
    finally:
        c.close()
