"""GPU parity: preemptible causal prefill attention through the C ABI against the fp64 oracle."""
import numpy as np
import pytest
import torch

import synth
from oracle.plan import prefill_plan
from oracle.prefill import paged_prefill_attention

pytestmark = pytest.mark.gpu

TOL = 1e-2


def make(name, seed, q_lens, **over):
    from gpu_util import DeviceCase
    c = DeviceCase(synth.workload(name, **over), seed=seed)
    g = c.wl.geom
    q_len = np.minimum(np.asarray(q_lens, dtype=np.int64), c.st.ctx_len).astype(np.int32)
    q_start = np.concatenate([[0], np.cumsum(q_len)[:-1]]).astype(np.int32)
    total = int(q_len.sum())
    q = synth.hash_bf16_bits(np.arange(total * g.num_q_heads * g.head_dim, dtype=np.int64) + 7 * seed, seed, 1)
    q = q.reshape(total, g.num_q_heads, g.head_dim)
    return c, q, q_start, q_len


def run_prefill(c, q, q_len, layer, slice_bytes, chunk_tokens, through_scheduler=False):
    vkv, g = c.vkv, c.wl.geom
    info = vkv.kv_prefill_plan(c.pool, c.st.ctx_len, q_len, slice_bytes, chunk_tokens)
    ws = torch.empty(info.workspace_bytes, dtype=torch.uint8, device="cuda:0")
    vkv.kv_prefill_bind(c.pool, ws)
    q_t = torch.from_numpy(q.view(np.int16)).cuda()
    out = torch.full((info.total_q, g.num_q_heads, g.head_dim), float("nan"), dtype=torch.float32, device="cuda:0")
    if through_scheduler:
        st, cur = vkv.kv_prefill_run_layer(c.pool, layer, 0, q_t, c.tables_t, ws, out)
        assert (st, cur) == (vkv.VKV_OK, info.n_slices + info.n_merge_steps)
    else:
        for s in range(info.n_slices):
            vkv.paged_prefill_attn_slice(c.pool, layer, s, q_t, c.tables_t, ws, out)
        for step in range(info.n_merge_steps):
            vkv.kv_prefill_merge(c.pool, step, ws, out)
    vkv.kv_prefill_check(c.pool, ws)
    return info, out.cpu().numpy(), (ws, q_t)


@pytest.mark.parametrize("name,seed,q_lens,chunk,slice_bytes", [
    ("llama8b_small", 1, [1, 33, 300, 64, 5, 128, 4096, 17], 512, 1 << 20),
    ("llama8b_small", 2, [4096] * 8, 2048, 8 << 20),
    ("llama70b_tp8_small", 3, [100, 1, 16, 700, 31, 32, 33, 2000, 8, 9, 10, 640], 256, 1 << 19),
    ("offline_batch_small", 4, [1000, 2, 129, 4096, 77, 512], 1024, 1 << 21),
    # items of one, two and three token groups only: the start and the end of the kernel's pipeline over groups
    ("llama8b_small", 6, [64, 96, 33, 200, 1, 7, 130, 65], 32, 1 << 18),
    ("llama8b_small", 7, [64, 96, 33, 200, 1, 7, 130, 65], 64, 1 << 18),
    ("stress_small", 8, [96, 97, 31, 250, 2, 500, 64, 190, 32, 1], 96, 1 << 18),
    # items longer than two 64-entry windows of block ids
    ("llama70b_tp8_small", 5, [1500, 40, 8192, 3, 700, 2500, 64, 1, 900, 4000, 33, 256], 8192, 4 << 20),
])
def test_prefill_matches_oracle(name, seed, q_lens, chunk, slice_bytes):
    from gpu_util import layout_of
    c, q, q_start, q_len = make(name, seed, q_lens)
    try:
        g = c.wl.geom
        layer = g.num_layers - 1
        info, got, _ = run_prefill(c, q, q_len, layer, slice_bytes, chunk)
        want_plan = prefill_plan(c.st.ctx_len, q_len, g.num_q_heads, g.num_kv_heads, g.head_dim, g.block_tokens,
                                 chunk, slice_bytes)
        for a, b in zip(c.vkv.kv_prefill_plan_read(c.pool, info), want_plan):
            assert np.array_equal(a, b)
        ref = paged_prefill_attention(c.pool_bits, layout_of(g), q, q_start, q_len, c.st.tables, c.st.ctx_len, layer)
        assert np.isfinite(got).all()
        err = float(np.max(np.abs(got.astype(np.float64) - ref)))
        flops = sum(4.0 * g.head_dim * g.num_q_heads * (int(c.st.ctx_len[s]) - int(q_len[s]) + i + 1)
                    for s in range(len(q_len)) for i in range(int(q_len[s])))
        assert abs(info.flops_per_layer - flops) <= 1e-6 * flops
        print(f"{name}: rows {info.total_q} tiles {info.n_tiles} items {info.n_items} slices {info.n_slices} "
              f"max|err| {err:.3e}", flush=True)
        assert err <= TOL
        # the scheduler path (slices + merge) gives the same bits
        _, got2, _ = run_prefill(c, q, q_len, layer, slice_bytes, chunk, through_scheduler=True)
        assert np.array_equal(got, got2)
        # another partition of the same work: same result within fp32 noise
        _, got3, _ = run_prefill(c, q, q_len, layer, 1 << 30, 2048)
        assert float(np.max(np.abs(got3.astype(np.float64) - ref))) <= TOL
    finally:
        c.close()


@pytest.mark.parametrize("overlap", [False, True])
def test_prefill_yield_resume_and_reclaim_keep_the_bits(overlap):
    c, q, q_start, q_len = make("stress_small", 6, [700, 64, 2048, 300, 1, 1500, 90, 1024, 33, 512])
    try:
        vkv, g = c.vkv, c.wl.geom
        vkv.kv_sched_set_overlap(c.pool, overlap)
        info, full, (ws, q_t) = run_prefill(c, q, q_len, 1, 1 << 20, 512)
        assert info.n_slices >= 6
        out = torch.empty((info.total_q, g.num_q_heads, g.head_dim), dtype=torch.float32, device="cuda:0")
        n, m = info.n_slices, info.n_merge_steps
        assert m >= 3                               # the merge is cut into steps too
        # a yield pending before slice k (k < n) or before merge step k - n
        for k in (0, n // 2, n - 1, n, n + m // 2, n + m - 1):
            out.fill_(float("nan"))
            for s in range(min(k, n)):
                vkv.paged_prefill_attn_slice(c.pool, 1, s, q_t, c.tables_t, ws, out)
            for t in range(max(0, k - n)):
                vkv.kv_prefill_merge(c.pool, t, ws, out)
            vkv.kv_yield_request(c.pool)
            st, cur = vkv.kv_prefill_run_layer(c.pool, 1, k, q_t, c.tables_t, ws, out)
            assert (st, cur) == (vkv.VKV_YIELDED, k)
            vkv.kv_yield_clear(c.pool)
            if k == info.n_slices // 2:
                # memory is reclaimed while the prefill is parked; the online tenant scribbles on it
                lo, hi = c.wl.reclaim_range
                stats = vkv.kv_reclaim_range(c.pool, lo, hi, c.tables_t, c.remap_t)
                assert stats.blocks_moved > 0
                c.pool_t.view(g.num_blocks, g.block_elems)[lo:hi] = synth.BF16_NAN_BITS
            st, cur = vkv.kv_prefill_run_layer(c.pool, 1, cur, q_t, c.tables_t, ws, out)
            assert (st, cur) == (vkv.VKV_OK, info.n_slices + info.n_merge_steps)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy(), full), f"resume at slice {k}"
    finally:
        c.close()


def test_prefill_rejects_bad_arguments():
    c, q, q_start, q_len = make("llama8b_small", 8, [10] * 8)
    try:
        vkv = c.vkv
        bad = q_len.copy()
        bad[3] = 0
        with pytest.raises(vkv.VkvError) as ei:
            vkv.kv_prefill_plan(c.pool, c.st.ctx_len, bad, 1 << 20, 512)
        assert ei.value.code == vkv.VKV_E_INVAL
        bad[3] = int(c.st.ctx_len[3]) + 1
        with pytest.raises(vkv.VkvError):
            vkv.kv_prefill_plan(c.pool, c.st.ctx_len, bad, 1 << 20, 512)
        with pytest.raises(vkv.VkvError):
            vkv.kv_prefill_plan(c.pool, c.st.ctx_len, q_len, 1 << 20, 100)
        info = vkv.kv_prefill_plan(c.pool, c.st.ctx_len, q_len, 1 << 20, 512)
        ws = torch.empty(info.workspace_bytes, dtype=torch.uint8, device="cuda:0")
        out = torch.empty((info.total_q, 32, 128), dtype=torch.float32, device="cuda:0")
        q_t = torch.from_numpy(q.view(np.int16)).cuda()
        with pytest.raises(vkv.VkvError) as ei:                     # not bound yet
            vkv.paged_prefill_attn_slice(c.pool, 0, 0, q_t, c.tables_t, ws, out)
        assert ei.value.code == vkv.VKV_E_STATE
        vkv.kv_prefill_bind(c.pool, ws)
        with pytest.raises(vkv.VkvError):
            vkv.paged_prefill_attn_slice(c.pool, 0, info.n_slices, q_t, c.tables_t, ws, out)
        with pytest.raises(vkv.VkvError):
            vkv.paged_prefill_attn_slice(c.pool, 9, 0, q_t, c.tables_t, ws, out)
    finally:
        c.close()
