"""The bandwidth yardsticks run, leave their inputs alone and reject bad arguments."""
import pytest

pytestmark = pytest.mark.gpu


def test_probe_read_and_copy():
    import torch
    import paper_2604_07874_amd as vkv
    dev = torch.device("cuda:0")
    n = 16 * 1000003                       # not a multiple of the 64 KiB a workgroup reads
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device=dev)
    keep = src.clone()
    sink = torch.zeros(256, dtype=torch.uint8, device=dev)
    vkv.kv_probe_read(src, n, sink)
    dst = torch.zeros_like(src)
    vkv.kv_probe_copy(dst, src, n)
    torch.cuda.synchronize()
    assert torch.equal(src, keep) and torch.equal(dst, keep)
    assert int(sink.sum()) == 0
    for bad in (0, 24):
        with pytest.raises(vkv.VkvError) as ei:
            vkv.kv_probe_read(src, bad, sink)
        assert ei.value.code == vkv.VKV_E_INVAL


def test_probe_attention_reads_runs_over_a_bound_plan():
    import numpy as np
    import torch
    import synth
    from gpu_util import DeviceCase
    c = DeviceCase(synth.workload("llama8b_small"), 3)
    try:
        vkv = c.vkv
        info = c.plan(slice_bytes=1 << 20)
        before = c.pool_t.clone()
        sink = torch.zeros(256, dtype=torch.uint8, device="cuda:0")
        for layer in range(c.wl.geom.num_layers):
            for s in range(info.n_slices):
                vkv.kv_probe_attn_reads(c.pool, layer, s, c.tables_t, c.ws, sink)
        vkv.kv_attn_check(c.pool, c.ws)
        assert torch.equal(c.pool_t, before) and int(sink.sum()) == 0
        with pytest.raises(vkv.VkvError) as ei:
            vkv.kv_probe_attn_reads(c.pool, 0, info.n_slices, c.tables_t, c.ws, sink)
        assert ei.value.code == vkv.VKV_E_INVAL
    finally:
        c.close()


def test_launch_timing_records_are_sane_and_leave_the_bits_alone():
    """Recording on: every slice launch carries its own start/stop events; the records name the slices in
    order, their durations are positive and add up to no more than the pass took, sampling thins them
    out, and the outputs are the bits of an unrecorded pass."""
    import time
    import numpy as np
    import torch
    import synth
    from gpu_util import DeviceCase
    c = DeviceCase(synth.workload("stress_small"), 9)
    try:
        vkv, g = c.vkv, c.wl.geom
        info = c.plan(slice_bytes=1 << 19)
        assert info.n_slices >= 8
        q, q_t = c.q_dev(0)
        plain = c.attention(0, q_t)
        out = torch.empty((c.wl.num_seqs, g.num_q_heads, g.head_dim), dtype=torch.float32, device="cuda:0")
        stream = torch.cuda.current_stream()
        vkv.kv_profile_enable(c.pool, 4 * info.n_slices)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        st, cur = vkv.kv_attn_run_layer(c.pool, 0, 0, q_t, c.tables_t, c.ws, out, max_inflight=2, stream=stream)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        assert (st, cur) == (vkv.VKV_OK, info.n_slices)
        rec = vkv.kv_profile_read(c.pool, 1 << 12)
        assert len(rec) == info.n_slices and (rec["kind"] == vkv.VKV_PROF_SLICE).all()
        assert rec["index"].tolist() == list(range(info.n_slices))
        assert (rec["ms"] > 0).all() and float(rec["ms"].sum()) <= wall_ms
        assert np.array_equal(out.cpu().numpy(), plain)
        vkv.kv_profile_sample(c.pool, 3)
        vkv.kv_attn_run_layer(c.pool, 0, 0, q_t, c.tables_t, c.ws, out, max_inflight=2, stream=stream)
        rec = vkv.kv_profile_read(c.pool, 1 << 12)
        assert len(rec) == -(-info.n_slices // 3) and (rec["ms"] > 0).all()
        vkv.kv_profile_enable(c.pool, 0)
        assert np.array_equal(out.cpu().numpy(), plain)
    finally:
        c.close()
