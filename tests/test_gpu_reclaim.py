"""GPU parity: KV reclamation (block relocation + table rewrite) against the oracle, bit for bit,
and the invariance of attention under reclamation and under yield/resume."""
import threading
import time

import numpy as np
import pytest
import torch

import synth
from oracle import reclaim as R
from oracle.attention import paged_decode_attention

pytestmark = pytest.mark.gpu


def make_case(name, seed, **over):
    from gpu_util import DeviceCase
    return DeviceCase(synth.workload(name, **over), seed=seed)


def oracle_for(c):
    g = c.wl.geom
    pool = c.pool_bits.reshape(g.num_blocks, g.block_elems).copy()
    return R.ReclaimOracle(g.num_blocks, g.blocks_per_handle, c.st.live, c.st.tables, pool)


def compare_state(c, orc, lo_hi_released):
    """Device pool / tables / live / ranges equal the oracle's, except bytes inside released ranges."""
    g = c.wl.geom
    torch.cuda.synchronize()
    live, ranges = c.vkv.kv_pool_state(c.pool, g.num_blocks)
    assert np.array_equal(live, orc.live)
    assert sorted(ranges) == sorted(orc.released) == sorted(lo_hi_released)
    tables = c.tables_t.cpu().numpy()
    assert np.array_equal(tables, orc.tables)
    c.vkv.kv_pool_check_tables(c.pool, tables)
    dev = c.pool_t.cpu().numpy().view(np.uint16).reshape(g.num_blocks, g.block_elems)
    keep = np.ones(g.num_blocks, dtype=bool)
    for lo, hi in lo_hi_released:
        keep[lo:hi] = False
    assert np.array_equal(dev[keep], orc.pool[keep])


@pytest.mark.parametrize("name,seed,over", [
    ("tiny", 0, {}),
    ("tiny", 3, {"shared_prefix_blocks": 1, "ctx_dist": ("uniform", 40, 256)}),
    ("llama8b_small", 1, {}),
    ("llama70b_tp8_small", 2, {}),
    ("stress_small", 4, {}),
])
def test_reclaim_matches_oracle(name, seed, over):
    c = make_case(name, seed, **over)
    try:
        g = c.wl.geom
        orc = oracle_for(c)
        lo, hi = c.wl.reclaim_range
        remap_plan, st_plan = c.vkv.kv_reclaim_plan(c.pool, lo, hi, g.num_blocks)
        stats = c.vkv.kv_reclaim_range(c.pool, lo, hi, c.tables_t, c.remap_t, chunk_bytes=c.wl.chunk_bytes)
        status, src, dst, remap = orc.reclaim(lo, hi)
        assert status == R.OK
        assert stats.blocks_moved == len(src) == st_plan.blocks_moved and len(src) > 0
        assert stats.bytes_moved == len(src) * g.block_bytes and stats.blocks_in_range == hi - lo
        assert stats.n_chunks == -(-len(src) // max(1, c.wl.chunk_bytes // g.block_bytes))
        assert np.array_equal(c.remap_t.cpu().numpy(), remap) and np.array_equal(remap_plan, remap)
        compare_state(c, orc, [(lo, hi)])
        # the same range again: refused, nothing changes
        with pytest.raises(c.vkv.VkvError) as ei:
            c.vkv.kv_reclaim_range(c.pool, lo, hi, c.tables_t, c.remap_t)
        assert ei.value.code == c.vkv.VKV_E_BUSY
        compare_state(c, orc, [(lo, hi)])
        # a second, lower range (single launch), then give the first one back and reclaim it again
        lo2 = lo - 2 * g.blocks_per_handle
        status2 = orc.reclaim(lo2, lo)[0]
        held = [(lo, hi)]
        if status2 == R.OK:
            c.vkv.kv_reclaim_range(c.pool, lo2, lo, c.tables_t, c.remap_t, chunk_bytes=0)
            held.append((lo2, lo))
        else:                       # a crowded pool: both sides must refuse alike
            with pytest.raises(c.vkv.VkvError) as ei:
                c.vkv.kv_reclaim_range(c.pool, lo2, lo, c.tables_t, c.remap_t, chunk_bytes=0)
            assert ei.value.code == status2 == R.E_NOSPACE
        compare_state(c, orc, held)
        c.vkv.kv_pool_return_range(c.pool, lo, hi)
        assert orc.return_range(lo, hi) == R.OK
        stats = c.vkv.kv_reclaim_range(c.pool, lo, hi, c.tables_t, c.remap_t)
        assert orc.reclaim(lo, hi)[0] == R.OK and stats.blocks_moved == 0
        compare_state(c, orc, held[1:] + [(lo, hi)])
        # with the high range returned, a low range can move up into it
        c.vkv.kv_pool_return_range(c.pool, lo, hi)
        assert orc.return_range(lo, hi) == R.OK
        bph = g.blocks_per_handle
        stats = c.vkv.kv_reclaim_range(c.pool, 0, bph, c.tables_t, c.remap_t, chunk_bytes=c.wl.chunk_bytes)
        status3, src3, dst3, remap3 = orc.reclaim(0, bph)
        assert status3 == R.OK and stats.blocks_moved == len(src3)
        assert np.array_equal(c.remap_t.cpu().numpy(), remap3)
        compare_state(c, orc, held[1:] + [(0, bph)])
    finally:
        c.close()


def test_error_paths_leave_everything_untouched():
    c = make_case("tiny", 5)
    try:
        g = c.wl.geom
        orc = oracle_for(c)
        for lo, hi, code in [(-8, 8, c.vkv.VKV_E_INVAL), (8, 8, c.vkv.VKV_E_INVAL), (4, 16, c.vkv.VKV_E_INVAL),
                             (248, 264, c.vkv.VKV_E_INVAL), (0, 200, c.vkv.VKV_E_NOSPACE)]:
            with pytest.raises(c.vkv.VkvError) as ei:
                c.vkv.kv_reclaim_range(c.pool, lo, hi, c.tables_t, c.remap_t)
            assert ei.value.code == code
            assert orc.reclaim(lo, hi)[0] == code   # the oracle's codes carry the same numbers
            compare_state(c, orc, [])
    finally:
        c.close()


def test_block_table_rewrite_alone():
    c = make_case("tiny", 6)
    try:
        nb = c.wl.geom.num_blocks
        rng = np.random.default_rng(0)
        remap = rng.permutation(nb).astype(np.int32)
        tables = rng.integers(-1, nb, size=(37, 19)).astype(np.int32)
        t_dev = torch.from_numpy(tables).cuda()
        c.vkv.block_table_rewrite(t_dev, torch.from_numpy(remap).cuda(), nb)
        expect = np.where(tables >= 0, remap[np.maximum(tables, 0)], tables)
        assert np.array_equal(t_dev.cpu().numpy(), expect)
    finally:
        c.close()


def test_attention_unchanged_by_reclaim_and_poison():
    from gpu_util import layout_of
    c = make_case("llama8b_small", 7)
    try:
        g = c.wl.geom
        c.plan()
        q, q_t = c.q_dev(1)
        before = c.attention(1, q_t)
        ref = paged_decode_attention(c.pool_bits, layout_of(g), q, c.st.tables, c.st.ctx_len, 1)
        assert np.max(np.abs(before - ref)) <= 1e-2
        lo, hi = c.wl.reclaim_range
        stats = c.vkv.kv_reclaim_range(c.pool, lo, hi, c.tables_t, c.remap_t, chunk_bytes=c.wl.chunk_bytes)
        assert stats.blocks_moved > 0
        # the online tenant overwrites its new memory: bf16 NaN everywhere in the range
        c.pool_t.view(g.num_blocks, g.block_elems)[lo:hi] = synth.BF16_NAN_BITS
        after = c.attention(1, q_t)
        assert np.isfinite(after).all()
        assert np.array_equal(before, after)      # the work partition is by position: bitwise equal
    finally:
        c.close()


@pytest.mark.parametrize("overlap", [False, True])
def test_yield_resume_is_bit_identical_at_every_slice(overlap):
    c = make_case("offline_batch_small", 8)
    try:
        g, vkv = c.wl.geom, c.vkv
        vkv.kv_sched_set_overlap(c.pool, overlap)   # every other slice on the pool's second stream
        info = c.plan(slice_bytes=1 << 20)
        assert info.n_slices >= 8
        q, q_t = c.q_dev(0)
        full = c.attention(0, q_t)
        out = torch.empty((c.wl.num_seqs, g.num_q_heads, g.head_dim), dtype=torch.float32, device="cuda:0")
        # uninterrupted run through the scheduler
        st, cur = vkv.kv_attn_run_layer(c.pool, 0, 0, q_t, c.tables_t, c.ws, out)
        assert (st, cur) == (vkv.VKV_OK, info.n_slices)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), full)
        # a yield request pending before slice k: stop there, resume, same bits
        for k in range(info.n_slices):
            out.fill_(float("nan"))
            # run slices [0,k) one by one, then request the yield
            for s in range(k):
                vkv.paged_decode_attn_slice(c.pool, 0, s, q_t, c.tables_t, c.ws, out)
            vkv.kv_yield_request(c.pool)
            st, cur = vkv.kv_attn_run_layer(c.pool, 0, k, q_t, c.tables_t, c.ws, out)
            assert (st, cur) == (vkv.VKV_YIELDED, k) and vkv.kv_yield_pending(c.pool)
            vkv.kv_yield_clear(c.pool)
            st, cur = vkv.kv_attn_run_layer(c.pool, 0, cur, q_t, c.tables_t, c.ws, out)
            assert (st, cur) == (vkv.VKV_OK, info.n_slices)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy(), full), f"resume at slice {k}"
        # the layers above began slice by slice (every chunk counted where it ran) and were finished by the
        # scheduler, which merges a layer of this many slices behind its last slice: no count may be left
        # over for the next layer, run slice by slice on the same workspace
        q1, q1_t = c.q_dev(1)
        got1 = c.attention(1, q1_t)
        vkv.kv_attn_bind(c.pool, c.ws)               # counters zeroed
        assert np.array_equal(c.attention(1, q1_t), got1)
    finally:
        c.close()


def test_reclaim_between_slices_keeps_attention_bitwise():
    c = make_case("stress_small", 9)
    try:
        g, vkv = c.wl.geom, c.vkv
        info = c.plan(slice_bytes=1 << 20)
        q, q_t = c.q_dev(1)
        full = c.attention(1, q_t)
        lo, hi = c.wl.reclaim_range
        out = torch.empty((c.wl.num_seqs, g.num_q_heads, g.head_dim), dtype=torch.float32, device="cuda:0")
        k = info.n_slices // 2
        for s in range(k):
            vkv.paged_decode_attn_slice(c.pool, 1, s, q_t, c.tables_t, c.ws, out)
        copy_stream = torch.cuda.Stream()
        stats = vkv.kv_reclaim_range(c.pool, lo, hi, c.tables_t, c.remap_t, chunk_bytes=c.wl.chunk_bytes,
                                     copy_stream=copy_stream, decode_stream=torch.cuda.current_stream())
        assert stats.blocks_moved > 0
        c.pool_t.view(g.num_blocks, g.block_elems)[lo:hi] = synth.BF16_NAN_BITS
        st, cur = vkv.kv_attn_run_layer(c.pool, 1, k, q_t, c.tables_t, c.ws, out)
        assert st == vkv.VKV_OK
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), full)
    finally:
        c.close()


def test_yield_from_another_thread_lands_and_resumes():
    c = make_case("offline_batch_small", 10)
    try:
        g, vkv = c.wl.geom, c.vkv
        info = c.plan(slice_bytes=64 << 10)      # many short slices
        q, q_t = c.q_dev(0)
        full = c.attention(0, q_t)
        out = torch.empty((c.wl.num_seqs, g.num_q_heads, g.head_dim), dtype=torch.float32, device="cuda:0")
        stream = torch.cuda.current_stream()
        timer = threading.Timer(0.002, lambda: vkv.kv_yield_request(c.pool))
        timer.start()
        cur, yields = 0, 0
        deadline = time.time() + 30
        while time.time() < deadline:
            st, cur = vkv.kv_attn_run_layer(c.pool, 0, cur, q_t, c.tables_t, c.ws, out, stream=stream)
            if st == vkv.VKV_OK:
                break
            yields += 1
            assert stream.query()                  # offline compute is off the GPU when the call returns
            vkv.kv_yield_clear(c.pool)
        timer.join()
        assert st == vkv.VKV_OK and cur == info.n_slices
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), full)
        print(f"slices {info.n_slices}, yields honoured {yields}", flush=True)
    finally:
        c.close()


def test_rate_cap_is_respected():
    c = make_case("offline_batch_small", 11, occupancy=0.8)
    try:
        g, vkv = c.wl.geom, c.vkv
        orc = oracle_for(c)
        lo, hi = c.wl.reclaim_range
        cap = 2e9
        stats = vkv.kv_reclaim_range(c.pool, lo, hi, c.tables_t, c.remap_t, chunk_bytes=2 << 20,
                                     rate_cap_bytes_per_s=int(cap))
        assert orc.reclaim(lo, hi)[0] == R.OK
        compare_state(c, orc, [(lo, hi)])
        assert stats.n_chunks >= 8
        # launch j waits until the bytes of launches < j fit under the cap
        floor = (stats.bytes_moved - (2 << 20)) / cap
        assert stats.host_seconds >= floor
        assert stats.bytes_moved / stats.host_seconds <= cap * 1.0 * stats.n_chunks / (stats.n_chunks - 1) * 1.001
        assert stats.host_seconds <= floor * 1.25 + 0.05     # and it is not much slower than the cap allows
        print(f"moved {stats.bytes_moved / 1e6:.1f} MB in {stats.host_seconds * 1e3:.1f} ms "
              f"({stats.bytes_moved / stats.host_seconds / 1e9:.2f} GB/s, cap {cap / 1e9} GB/s)", flush=True)
    finally:
        c.close()


@pytest.mark.parametrize("overlap", [False, True])
def test_rate_capped_reclaim_while_decode_runs_on_another_stream(overlap):
    """The offline-batch shape's scenario: decode keeps running on its stream (its own host thread)
    while the range is emptied in small launches under a rate cap on a second stream."""
    c = make_case("offline_batch_small", 12, occupancy=0.8)
    try:
        g, vkv = c.wl.geom, c.vkv
        vkv.kv_sched_set_overlap(c.pool, overlap)   # before the second thread exists
        orc = oracle_for(c)
        info = c.plan(slice_bytes=1 << 20)
        L = g.num_layers
        qs = [c.q_dev(l)[1] for l in range(L)]
        base = [torch.from_numpy(c.attention(l, qs[l])).cuda() for l in range(L)]
        decode_stream, copy_stream = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        stop = threading.Event()
        result = {"passes": 0, "bad": 0, "error": None}

        def decode_loop():
            try:
                out = torch.empty_like(base[0])
                with torch.cuda.stream(decode_stream):
                    while not stop.is_set() or result["passes"] < 3:
                        for l in range(L):
                            out.fill_(float("nan"))
                            st_, cur = vkv.kv_attn_run_layer(c.pool, l, 0, qs[l], c.tables_t, c.ws, out,
                                                             stream=decode_stream)
                            assert st_ == vkv.VKV_OK
                            decode_stream.synchronize()
                            if not torch.equal(out, base[l]):
                                result["bad"] += 1
                        result["passes"] += 1
            except Exception as e:          # surfaced by the main thread
                result["error"] = e

        th = threading.Thread(target=decode_loop)
        th.start()
        time.sleep(0.01)
        lo, hi = c.wl.reclaim_range
        cap = 1e9
        stats = vkv.kv_reclaim_range(c.pool, lo, hi, c.tables_t, c.remap_t, chunk_bytes=1 << 20,
                                     rate_cap_bytes_per_s=int(cap), copy_stream=copy_stream,
                                     decode_stream=decode_stream)
        passes_during = result["passes"]
        # the online tenant overwrites its range while decode goes on
        with torch.cuda.stream(copy_stream):
            c.pool_t.view(g.num_blocks, g.block_elems)[lo:hi] = synth.BF16_NAN_BITS
        copy_stream.synchronize()
        time.sleep(0.02)
        stop.set()
        th.join(timeout=60)
        assert not th.is_alive() and result["error"] is None, result["error"]
        assert result["bad"] == 0 and result["passes"] >= 3
        assert stats.n_chunks >= 16 and stats.host_seconds >= (stats.bytes_moved - (1 << 20)) / cap
        assert orc.reclaim(lo, hi)[0] == R.OK
        compare_state(c, orc, [(lo, hi)])
        vkv.kv_attn_check(c.pool, c.ws)
        print(f"{passes_during} decode passes finished while {stats.bytes_moved / 1e6:.1f} MB moved in "
              f"{stats.host_seconds * 1e3:.1f} ms; {result['passes']} passes in all, all bit-identical", flush=True)
    finally:
        c.close()
