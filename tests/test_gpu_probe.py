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
