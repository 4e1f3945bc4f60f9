"""GPU parity: paged decode attention through the C ABI against the fp64 oracle."""
import numpy as np
import pytest
import torch

import synth
from oracle.attention import paged_decode_attention
from oracle.plan import attention_plan

pytestmark = pytest.mark.gpu

TOL = 1e-2   # max-abs bound on fp32 outputs (bf16 K/V, fp32 accumulate)


@pytest.fixture(scope="module")
def tiny_case():
    from gpu_util import DeviceCase
    c = DeviceCase(synth.workload("tiny"), seed=0)
    yield c
    c.close()


def check_attention(c, layers, **plan_kw):
    from gpu_util import layout_of
    info = c.plan(**plan_kw)
    worst = 0.0
    for layer in layers:
        q, q_t = c.q_dev(layer)
        got = c.attention(layer, q_t)
        ref = paged_decode_attention(c.pool_bits, layout_of(c.wl.geom), q, c.st.tables, c.st.ctx_len, layer)
        assert np.isfinite(got).all()
        err = float(np.max(np.abs(got.astype(np.float64) - ref)))
        print(f"{c.wl.name} layer {layer}: items {info.n_items} slices {info.n_slices} max|err| {err:.3e}", flush=True)
        worst = max(worst, err)
    assert worst <= TOL
    return worst


def test_plan_matches_oracle(tiny_case):
    c = tiny_case
    g = c.wl.geom
    for chunk, sb in [(64, 256 << 10), (32, 1), (256, 1 << 30), (128, 40000)]:
        info = c.vkv.kv_attn_plan(c.pool, c.st.ctx_len, sb, chunk)
        work, starts = c.vkv.kv_attn_plan_read(c.pool, info)
        owork, ostarts = attention_plan(c.st.ctx_len, g.num_kv_heads, g.head_dim, g.block_tokens, chunk, sb)
        assert np.array_equal(work, owork) and np.array_equal(starts, ostarts)
        assert info.kv_bytes_per_layer == int(c.st.ctx_len.sum()) * g.kv_bytes_per_token_layer


def test_tiny_attention(tiny_case):
    check_attention(tiny_case, [0])


@pytest.mark.parametrize("chunk,slice_bytes", [(32, 1), (64, 1 << 30), (96, 30000), (256, 100000)])
def test_tiny_attention_any_partition(tiny_case, chunk, slice_bytes):
    check_attention(tiny_case, [0], chunk_tokens=chunk, slice_bytes=slice_bytes)


@pytest.mark.parametrize("name", ["llama8b_small", "llama70b_tp8_small", "offline_batch_small", "stress_small"])
def test_small_configs(name):
    from gpu_util import DeviceCase
    wl = synth.workload(name)
    c = DeviceCase(wl, seed=1)
    try:
        check_attention(c, range(wl.geom.num_layers))
        check_attention(c, [wl.geom.num_layers - 1], chunk_tokens=128, slice_bytes=1 << 20)
    finally:
        c.close()


def test_overlapped_slices_keep_stream_order_and_bits():
    """With every other slice on the pool's second stream, work enqueued on the caller's stream
    before the call still precedes all slices and work enqueued after it follows all of them."""
    from gpu_util import DeviceCase
    c = DeviceCase(synth.workload("stress_small"), 11)
    try:
        g, vkv = c.wl.geom, c.vkv
        info = c.plan(slice_bytes=1 << 19)
        assert info.n_slices >= 8
        q, q_t = c.q_dev(1)
        full = c.attention(1, q_t)
        vkv.kv_sched_set_overlap(c.pool, True)
        side = torch.cuda.Stream()
        out = torch.empty((c.wl.num_seqs, g.num_q_heads, g.head_dim), dtype=torch.float32, device="cuda:0")
        torch.cuda.synchronize()
        for rep in range(3):
            with torch.cuda.stream(side):
                q_late = torch.zeros_like(q_t)
                q_late.copy_(q_t)                     # the query arrives on the stream just before the call
                out.fill_(float("nan"))
                st, cur = vkv.kv_attn_run_layer(c.pool, 1, 0, q_late, c.tables_t, c.ws, out, max_inflight=4, stream=side)
                assert (st, cur) == (vkv.VKV_OK, info.n_slices)
                got = out.clone()                     # read on the same stream right after, no host wait between
            side.synchronize()
            assert np.array_equal(got.cpu().numpy(), full), rep
        vkv.kv_attn_check(c.pool, c.ws, side)
    finally:
        c.close()


@pytest.mark.parametrize("pieces", ["many", "three"])
def test_merge_is_repeatable_when_chunks_of_a_sequence_arrive_from_many_launches(pieces):
    """32 chunks per sequence, cut into slices so that the chunks of one (sequence, kv head) finish in
    different launches running side by side on two streams.  In three slices whichever workgroup arrives
    last merges, inside the launches; in many slices (far smaller than a sequence) the scheduler has the
    layer merged once behind its last slice.  Twenty passes must give the bits of the one-launch result."""
    from gpu_util import DeviceCase
    wl = synth.workload("offline_batch_small", ctx_dist=("uniform", 3969, 4096))
    c = DeviceCase(wl, seed=47)
    try:
        g, vkv = wl.geom, c.vkv
        assert int(np.ceil(c.st.ctx_len / 128).min()) == 32
        q, q_t = c.q_dev(0)
        one = c.plan(slice_bytes=1 << 40, chunk_tokens=128)
        assert one.n_slices == 1
        ref = c.attention(0, q_t)
        if pieces == "many":
            many = c.plan(slice_bytes=1 << 20, chunk_tokens=128)
            assert many.n_slices >= 64 and many.n_items == one.n_items
        else:
            many = c.plan(slice_bytes=one.kv_bytes_per_layer // 3 + (1 << 16), chunk_tokens=128)
            assert many.n_slices == 3 and many.n_items == one.n_items
        vkv.kv_sched_set_overlap(c.pool, True)
        stream = torch.cuda.Stream()
        out = torch.empty((wl.num_seqs, g.num_q_heads, g.head_dim), dtype=torch.float32, device="cuda:0")
        for rep in range(20):
            with torch.cuda.stream(stream):
                out.fill_(float("nan"))
                st, cur = vkv.kv_attn_run_layer(c.pool, 0, 0, q_t, c.tables_t, c.ws, out, max_inflight=4, stream=stream)
            stream.synchronize()
            assert (st, cur) == (vkv.VKV_OK, many.n_slices)
            assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32)), f"pass {rep}"
        vkv.kv_attn_check(c.pool, c.ws, stream)
    finally:
        c.close()


def test_hand_derived_exact_cases_through_the_library():
    """The exact-rational cases of tests/golden/attention_exact_cases.json, embedded in head_dim 128
    (extra dimensions zero), through the decode and the prefill kernels: checks the library against
    hand-derived values, not against the oracle."""
    import json
    import math
    import os
    from fractions import Fraction
    import paper_2604_07874_amd as vkv
    from oracle.attention import PoolLayout
    fix = json.load(open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "attention_exact_cases.json")))
    gg = fix["geometry"]
    D, d0 = 128, gg["head_dim"]
    lay = PoolLayout(1, gg["num_kv_heads"], D, 16)
    nb = 4                                            # one handle of 4 blocks; block 3 stays free

    def bf16(x):
        u = np.asarray(x, dtype=np.float32).view(np.uint32)
        return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)

    pool = np.full(nb * lay.block_elems, synth.BF16_NAN_BITS, dtype=np.uint16)
    for blk, kv, head, slot, vals in fix["pool_entries"]:
        o = lay.vec_offset(blk, 0, kv, head, slot)
        pool[o:o + D] = 0
        pool[o:o + d0] = bf16(vals)
    pool_t = torch.from_numpy(pool.view(np.int16)).cuda()
    tables = np.array(fix["tables"], dtype=np.int32)
    tables_t = torch.from_numpy(tables).cuda()
    ctx = np.array(fix["ctx_len"], dtype=np.int32)
    p = vkv.kv_pool_init(1, gg["num_q_heads"], gg["num_kv_heads"], D, nb, 4, base=pool_t)
    vkv.kv_pool_adopt(p, np.array([0, 1, 2], dtype=np.int32))
    scales = {"ln2": math.log(2.0), "ln3": math.log(3.0)}
    try:
        info = vkv.kv_attn_plan(p, ctx, 1 << 20, 32)
        ws = torch.empty(info.workspace_bytes, dtype=torch.uint8, device="cuda:0")
        vkv.kv_attn_bind(p, ws)
        for case in fix["decode"]:
            q = np.zeros((2, gg["num_q_heads"], D), dtype=np.float32)
            q[:, :, :d0] = np.array(case["q"], dtype=np.float32)
            q_t = torch.from_numpy(bf16(q).view(np.int16)).cuda()
            out = torch.full((2, gg["num_q_heads"], D), float("nan"), dtype=torch.float32, device="cuda:0")
            st, cur = vkv.kv_attn_run_layer(p, 0, 0, q_t, tables_t, ws, out, softmax_scale=scales[case["scale"]])
            assert st == vkv.VKV_OK
            vkv.kv_attn_check(p, ws)
            got = out.cpu().numpy()
            want = np.array([[[float(Fraction(x)) for x in head] for head in seq] for seq in case["expect"]])
            assert np.max(np.abs(got[:, :, :d0] - want)) <= TOL, case["name"]
            assert np.all(got[:, :, d0:] == 0.0)
        for case in fix["prefill"]:
            q_len = np.array([case["q_len"][0], 1], dtype=np.int32)      # the library wants q_len >= 1 everywhere
            q = np.zeros((int(q_len.sum()), gg["num_q_heads"], D), dtype=np.float32)
            q[:q_len[0], :, :d0] = np.array(case["q_seq0"], dtype=np.float32)
            q_t = torch.from_numpy(bf16(q).view(np.int16)).cuda()
            pinfo = vkv.kv_prefill_plan(p, ctx, q_len, 1 << 20, 32)
            pws = torch.empty(pinfo.workspace_bytes, dtype=torch.uint8, device="cuda:0")
            vkv.kv_prefill_bind(p, pws)
            out = torch.full((pinfo.total_q, gg["num_q_heads"], D), float("nan"), dtype=torch.float32, device="cuda:0")
            st, cur = vkv.kv_prefill_run_layer(p, 0, 0, q_t, tables_t, pws, out, softmax_scale=scales[case["scale"]])
            assert st == vkv.VKV_OK
            vkv.kv_prefill_check(p, pws)
            got = out.cpu().numpy()
            want = np.array([[float(Fraction(x)) for x in row] for row in case["expect_seq0"]])
            for head in range(gg["num_q_heads"]):
                assert np.max(np.abs(got[:q_len[0], head, :d0] - want)) <= TOL, case["name"]
    finally:
        vkv.kv_pool_destroy(p)


def test_context_lengths_on_every_boundary():
    """Contexts of one token, around a block (16), a group (32), a chunk and the table-window (1024)
    boundaries, through chunked and unchunked plans."""
    from gpu_util import DeviceCase, layout_of
    wl = synth.workload("stress_small", ctx_dist=("uniform", 2049, 2049), num_seqs=10)
    c = DeviceCase(wl, seed=13)
    try:
        g = wl.geom
        q, q_t = c.q_dev(0)
        lay = layout_of(g)
        lengths = [1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 255, 256, 257, 511, 512, 513, 1023, 1024, 1025, 2047, 2048,
                   2049, 1, 100, 1000, 7, 2000, 48, 1536]
        assert int(c.st.ctx_len.min()) >= 2049
        for first in range(0, len(lengths), wl.num_seqs):
            ctx = np.array(lengths[first:first + wl.num_seqs], dtype=np.int32)
            want = paged_decode_attention(c.pool_bits, lay, q, c.st.tables, ctx, 0)
            for chunk, slice_bytes in ((2048, 1 << 30), (256, 1 << 18), (32, 1 << 14)):
                c.plan(slice_bytes=slice_bytes, chunk_tokens=chunk, ctx=ctx)
                got = c.attention(0, q_t)
                err = float(np.max(np.abs(got.astype(np.float64) - want)))
                assert err <= TOL, (ctx.tolist(), chunk, err)
    finally:
        c.close()
