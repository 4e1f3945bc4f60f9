"""GPU test of the entry point that allocates nothing: paged_decode_attn_layer_static keeps its
scratch in an array of the library's device image instead of a caller-provided workspace.

Its output must equal, bit for bit, what the planned path (kv_attn_plan / kv_attn_bind /
paged_decode_attn_slice) gives for the same chunk_tokens, and both must be within the attention
tolerance of the fp64 oracle.  Two calls in a row, the second with a smaller batch and shorter
sequences, so that whatever the first call left in the shared scratch is met by the second.
"""
import numpy as np
import pytest
import torch

import synth
from oracle.attention import paged_decode_attention

pytestmark = pytest.mark.gpu

TOL = 1e-2


def _planned(c, layer, q_t, ctx, chunk, slice_bytes):
    """Output of the existing entry points for the sequences ctx describes (rows 0..len(ctx)-1)."""
    g, vkv = c.wl.geom, c.vkv
    info = vkv.kv_attn_plan(c.pool, ctx, slice_bytes, chunk)
    ws = torch.empty(info.workspace_bytes, dtype=torch.uint8, device="cuda:0")
    vkv.kv_attn_bind(c.pool, ws)
    out = torch.full((len(ctx), g.num_q_heads, g.head_dim), float("nan"), dtype=torch.float32, device="cuda:0")
    for s in range(info.n_slices):
        vkv.paged_decode_attn_slice(c.pool, layer, s, q_t, c.tables_t, ws, out)
    vkv.kv_attn_check(c.pool, ws)
    return out


@pytest.mark.parametrize("name,chunk", [("llama8b_small", 256), ("tiny", 64)])
def test_static_entry_matches_planned_path_twice(name, chunk):
    from gpu_util import DeviceCase, layout_of
    wl = synth.workload(name)
    c = DeviceCase(wl, seed=5)
    try:
        g, vkv = wl.geom, c.vkv
        layer = g.num_layers - 1
        q, q_t = c.q_dev(layer)
        err_flag = torch.zeros(1, dtype=torch.int32, device="cuda:0")
        ctx_full = c.st.ctx_len.copy()
        # second call: fewer sequences, each shorter (and one of them a single token)
        n2 = max(2, wl.num_seqs // 2)
        ctx_small = np.maximum(1, ctx_full[:n2] // 3).astype(np.int32)
        ctx_small[0] = 1
        for ctx in (ctx_full, ctx_small):
            n = len(ctx)
            want = _planned(c, layer, q_t, ctx, chunk, 1 << 20)
            ctx_t = torch.from_numpy(ctx).to("cuda:0")
            got = torch.full((n, g.num_q_heads, g.head_dim), float("nan"), dtype=torch.float32, device="cuda:0")
            torch.cuda.synchronize()
            free_before = torch.cuda.mem_get_info()[0]
            reserved_before = torch.cuda.memory_reserved()
            vkv.paged_decode_attn_layer_static(c.pool, layer, q_t, c.tables_t, ctx_t, int(ctx.max()), chunk, got,
                                               err_flag_dev=err_flag)
            torch.cuda.synchronize()
            assert torch.cuda.mem_get_info()[0] == free_before and torch.cuda.memory_reserved() == reserved_before
            assert int(err_flag.item()) == 0
            assert torch.equal(got, want), f"{name}: static entry differs from the planned path ({n} sequences)"
            ref = paged_decode_attention(c.pool_bits, layout_of(g), q[:n], c.st.tables[:n], ctx, layer)
            err = float(np.max(np.abs(got.cpu().numpy().astype(np.float64) - ref)))
            print(f"{name}: {n} sequences, max ctx {int(ctx.max())}: bits equal, max|err| vs oracle {err:.2e}", flush=True)
            assert err <= TOL
    finally:
        c.close()


def test_static_entry_limits_and_flags():
    from gpu_util import DeviceCase
    wl = synth.workload("llama8b_small")
    c = DeviceCase(wl, seed=6, host_pool=False)
    try:
        g, vkv = wl.geom, c.vkv
        q, q_t = c.q_dev(0)
        n = wl.num_seqs
        ctx_t = torch.from_numpy(c.st.ctx_len).to("cuda:0")
        out = torch.zeros((n, g.num_q_heads, g.head_dim), dtype=torch.float32, device="cuda:0")
        # a batch whose partial results cannot fit the static array is refused before anything is enqueued
        big_tables = torch.full((4096, c.tables_t.shape[1]), -1, dtype=torch.int32, device="cuda:0")
        big_ctx = torch.ones(4096, dtype=torch.int32, device="cuda:0")
        big_q = torch.zeros((4096, g.num_q_heads, g.head_dim), dtype=torch.int16, device="cuda:0")
        big_out = torch.zeros((4096, g.num_q_heads, g.head_dim), dtype=torch.float32, device="cuda:0")
        with pytest.raises(vkv.VkvError) as e:
            vkv.paged_decode_attn_layer_static(c.pool, 0, big_q, big_tables, big_ctx, c.tables_t.shape[1] * 16, 32, big_out)
        assert e.value.code == vkv.VKV_E_NOSPACE and "static buffer" in str(e.value)
        # max_ctx_tokens beyond what the table can hold
        with pytest.raises(vkv.VkvError) as e:
            vkv.paged_decode_attn_layer_static(c.pool, 0, q_t, c.tables_t, ctx_t, c.tables_t.shape[1] * 16 + 1, 256, out)
        assert e.value.code == vkv.VKV_E_INVAL
        # a context length above the stated bound is clamped and flagged; the kernel stays inside the table
        flag = torch.zeros(1, dtype=torch.int32, device="cuda:0")
        bound = int(c.st.ctx_len.max()) // 2
        vkv.paged_decode_attn_layer_static(c.pool, 0, q_t, c.tables_t, ctx_t, bound, 256, out, err_flag_dev=flag)
        torch.cuda.synchronize()
        assert int(flag.item()) & 2
        # sequences within the bound are unaffected by the clamped ones
        ok = np.flatnonzero(c.st.ctx_len <= bound)
        assert len(ok) > 0
        want = torch.zeros_like(out)
        flag.zero_()
        vkv.paged_decode_attn_layer_static(c.pool, 0, q_t, c.tables_t, ctx_t, int(c.st.ctx_len.max()), 256, want,
                                           err_flag_dev=flag)
        torch.cuda.synchronize()
        assert int(flag.item()) == 0
        idx = torch.from_numpy(ok).to("cuda:0")
        assert torch.equal(out[idx], want[idx])
    finally:
        c.close()
