"""GPU parity on the kernel paths that the workload shapes do not reach by themselves: every group
size and head dimension the pool accepts, softmax inputs that force the running maximum to move
(a dominant key in every lane position, scores that rise along the sequence, logits of several
tens), block tables with bad entries, and blocks shared by two sequences.  Decode and prefill,
element-wise against the fp64 oracle, max-abs tolerance 1e-2."""
import math
from dataclasses import replace

import numpy as np
import pytest
import torch

import synth
from oracle.attention import PoolLayout, paged_decode_attention
from oracle.prefill import paged_prefill_attention

pytestmark = pytest.mark.gpu

TOL = 1e-2


def bf16_bits(x):
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


# ------------------------------------------------------------------ group sizes and head dims
@pytest.mark.parametrize("D,Hq,Hkv", [
    (64, 8, 4), (64, 16, 4), (64, 16, 2), (64, 16, 1), (64, 3, 1),
    (128, 4, 2), (128, 6, 2), (128, 12, 2), (128, 16, 1), (128, 5, 1), (128, 7, 1), (128, 2, 2)])
def test_every_group_size_and_head_dim(D, Hq, Hkv):
    """The pool accepts head_dim 64 or 128 and any group size up to 16: each of them against the oracle,
    with chunks short enough that results are merged across workgroups."""
    from gpu_util import DeviceCase, layout_of
    base = synth.workload("llama8b_small")
    geom = replace(base.geom, num_layers=2, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D, num_blocks=1024,
                   blocks_per_handle=32)
    wl = replace(base, geom=geom, num_seqs=6, ctx_dist=("uniform", 20, 900), reclaim_blocks=256)
    c = DeviceCase(wl, seed=Hq * 100 + Hkv)
    try:
        lay = layout_of(geom)
        for layer, chunk, sb in ((0, 128, 1 << 18), (1, 2048, 1 << 30), (1, 32, 1 << 16)):
            c.plan(slice_bytes=sb, chunk_tokens=chunk)
            q, q_t = c.q_dev(layer)
            got = c.attention(layer, q_t)
            ref = paged_decode_attention(c.pool_bits, lay, q, c.st.tables, c.st.ctx_len, layer)
            err = float(np.max(np.abs(got.astype(np.float64) - ref)))
            print(f"decode D={D} G={Hq // Hkv} chunk={chunk}: items {c.info.n_items} max|err| {err:.2e}", flush=True)
            assert np.isfinite(got).all() and err <= TOL
        if D == 128:      # the prefill kernel (head_dim 128 only; groups are padded to a power of two)
            vkv = c.vkv
            q_len = np.minimum(c.st.ctx_len, [64, 1, 300, 17, 900, 128]).astype(np.int32)
            q_start = np.concatenate([[0], np.cumsum(q_len)[:-1]]).astype(np.int32)
            total = int(q_len.sum())
            q = synth.hash_bf16_bits(np.arange(total * Hq * D, dtype=np.int64), 77, 1).reshape(total, Hq, D)
            info = vkv.kv_prefill_plan(c.pool, c.st.ctx_len, q_len, 1 << 19, 256)
            ws = torch.empty(info.workspace_bytes, dtype=torch.uint8, device="cuda:0")
            vkv.kv_prefill_bind(c.pool, ws)
            q_t = torch.from_numpy(q.view(np.int16)).cuda()
            out = torch.full((total, Hq, D), float("nan"), dtype=torch.float32, device="cuda:0")
            st, cur = vkv.kv_prefill_run_layer(c.pool, 1, 0, q_t, c.tables_t, ws, out)
            assert st == vkv.VKV_OK
            vkv.kv_prefill_check(c.pool, ws)
            ref = paged_prefill_attention(c.pool_bits, lay, q, q_start, q_len, c.st.tables, c.st.ctx_len, 1)
            err = float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - ref)))
            print(f"prefill G={Hq // Hkv}: rows {total} items {info.n_items} max|err| {err:.2e}", flush=True)
            assert err <= TOL
    finally:
        c.close()


# ------------------------------------------------------------------ crafted contents
class Crafted:
    """One-layer pool whose K and V rows are given as arrays: sequence s holds K[s], V[s] of shape
    [n_s, Hkv, D] (fp32 values, rounded to bf16 here); blocks are scattered by a seeded permutation;
    slots past a sequence's end hold NaN."""

    def __init__(self, K, V, Hq, seed=0):
        import paper_2604_07874_amd as vkv
        self.vkv = vkv
        S = len(K)
        Hkv, D = K[0].shape[1], K[0].shape[2]
        self.ctx = np.array([k.shape[0] for k in K], dtype=np.int32)
        nblk = -(-self.ctx // 16)
        nb = int(-(-int(nblk.sum()) // 8) * 8 + 8)
        self.lay = PoolLayout(1, Hkv, D, 16)
        rng = np.random.default_rng(seed)
        perm = rng.permutation(nb).astype(np.int32)
        self.tables = np.full((S, int(nblk.max())), -1, dtype=np.int32)
        pool = np.full((nb, 1, 2, Hkv, 16, D), synth.BF16_NAN_BITS, dtype=np.uint16)
        cur = 0
        for s in range(S):
            ids = perm[cur:cur + nblk[s]]
            cur += int(nblk[s])
            self.tables[s, :nblk[s]] = ids
            kb, vb = bf16_bits(K[s]), bf16_bits(V[s])
            for t in range(int(self.ctx[s])):
                pool[ids[t // 16], 0, 0, :, t % 16, :] = kb[t]
                pool[ids[t // 16], 0, 1, :, t % 16, :] = vb[t]
        self.pool_bits = pool.reshape(-1)
        self.pool_t = torch.from_numpy(self.pool_bits.view(np.int16)).cuda()
        self.tables_t = torch.from_numpy(self.tables).cuda()
        self.Hq, self.D, self.S = Hq, D, S
        self.pool = vkv.kv_pool_init(1, Hq, Hkv, D, nb, 8, base=self.pool_t)
        vkv.kv_pool_adopt(self.pool, np.sort(perm[:cur]))

    def close(self):
        self.vkv.kv_pool_destroy(self.pool)

    def decode(self, q, scale, chunk, slice_bytes):
        vkv = self.vkv
        info = vkv.kv_attn_plan(self.pool, self.ctx, slice_bytes, chunk)
        ws = torch.empty(info.workspace_bytes, dtype=torch.uint8, device="cuda:0")
        vkv.kv_attn_bind(self.pool, ws)
        qb = bf16_bits(q)
        q_t = torch.from_numpy(qb.view(np.int16)).cuda()
        out = torch.full((self.S, self.Hq, self.D), float("nan"), dtype=torch.float32, device="cuda:0")
        st, _ = vkv.kv_attn_run_layer(self.pool, 0, 0, q_t, self.tables_t, ws, out, softmax_scale=scale)
        assert st == vkv.VKV_OK
        vkv.kv_attn_check(self.pool, ws)
        ref = paged_decode_attention(self.pool_bits, self.lay, qb, self.tables, self.ctx, 0, scale=scale or None)
        return out.cpu().numpy(), ref

    def prefill(self, q_rows, q_len, scale, chunk, slice_bytes):
        vkv = self.vkv
        q_len = np.asarray(q_len, dtype=np.int32)
        q_start = np.concatenate([[0], np.cumsum(q_len)[:-1]]).astype(np.int32)
        info = vkv.kv_prefill_plan(self.pool, self.ctx, q_len, slice_bytes, chunk)
        ws = torch.empty(info.workspace_bytes, dtype=torch.uint8, device="cuda:0")
        vkv.kv_prefill_bind(self.pool, ws)
        qb = bf16_bits(q_rows)
        q_t = torch.from_numpy(qb.view(np.int16)).cuda()
        out = torch.full((int(q_len.sum()), self.Hq, self.D), float("nan"), dtype=torch.float32, device="cuda:0")
        st, _ = vkv.kv_prefill_run_layer(self.pool, 0, 0, q_t, self.tables_t, ws, out, softmax_scale=scale)
        assert st == vkv.VKV_OK
        vkv.kv_prefill_check(self.pool, ws)
        ref = paged_prefill_attention(self.pool_bits, self.lay, qb, q_start, q_len, self.tables, self.ctx, 0,
                                      scale=scale or None)
        return out.cpu().numpy(), ref


def test_dominant_key_in_every_lane_position():
    """One key far above the rest, in each of the 32 positions of a token group and in each position of
    the ragged last block: the output is that token's V row, and the running maximum has to jump to it
    wherever it sits in the lane layout."""
    rng = np.random.default_rng(3)
    Hq, Hkv, D, n = 8, 2, 128, 103             # three groups and a last block of 7 tokens
    positions = list(range(32, 64)) + list(range(96, 103))
    S = len(positions)
    q = rng.standard_normal((S, Hq, D)).astype(np.float32)
    q = bf16_bits(q).astype(np.uint32) << 16
    q = q.view(np.float32)                                     # the values the kernels will see
    K = [rng.standard_normal((n, Hkv, D)).astype(np.float32) for _ in range(S)]
    V = [rng.standard_normal((n, Hkv, D)).astype(np.float32) for _ in range(S)]
    for s, t in enumerate(positions):
        for h in range(Hkv):
            g0 = h * (Hq // Hkv)                               # the first query head of the group decides the direction
            K[s][t, h] = 45.0 * math.sqrt(D) * q[s, g0] / float(q[s, g0] @ q[s, g0])   # logit 45 for that head
    c = Crafted(K, V, Hq, seed=4)
    try:
        for chunk, sb in ((2048, 1 << 30), (32, 1 << 14)):
            got, ref = c.decode(q, 0.0, chunk, sb)
            err = float(np.max(np.abs(got.astype(np.float64) - ref)))
            print(f"dominant key, chunk {chunk}: max|err| {err:.2e}", flush=True)
            assert err <= TOL
            for s, t in enumerate(positions):                  # and it is that token's V row (bf16 values)
                for h in range(Hkv):
                    v = (bf16_bits(V[s][t, h]).astype(np.uint32) << 16).view(np.float32)
                    assert np.max(np.abs(got[s, h * (Hq // Hkv)] - v)) <= TOL
        # prefill: the same cache, the last 40 positions of every sequence as queries with the decode query's values
        q_len = np.full(S, 40, dtype=np.int32)
        q_rows = np.repeat(q, 40, axis=0)
        got, ref = c.prefill(q_rows, q_len, 0.0, 64, 1 << 16)
        err = float(np.max(np.abs(got.astype(np.float64) - ref)))
        print(f"dominant key, prefill: max|err| {err:.2e}", flush=True)
        assert err <= TOL
    finally:
        c.close()


def test_scores_rising_along_the_sequence_and_large_logits():
    """Scores that grow with the position make the running maximum move in every group of tokens (and
    push the prefill kernel's lazily updated reference over its slack again and again); a softmax
    scale that spreads the logits over +-60 tests the exponent range."""
    rng = np.random.default_rng(5)
    Hq, Hkv, D = 8, 2, 128
    lens = [2048, 1500, 777, 2048]
    S = len(lens)
    u = rng.standard_normal(D).astype(np.float32)
    u /= np.linalg.norm(u)
    q = (0.3 * rng.standard_normal((S, Hq, D)) + 4.0 * u).astype(np.float32)         # every query leans along u
    K, V = [], []
    for n in lens:
        k = 0.3 * rng.standard_normal((n, Hkv, D)).astype(np.float32)
        k += (0.14 * np.arange(n, dtype=np.float32))[:, None, None] * u               # q.k / sqrt(D) rises ~0.05 per token
        K.append(k.astype(np.float32))
        V.append(rng.standard_normal((n, Hkv, D)).astype(np.float32))
    c = Crafted(K, V, Hq, seed=6)
    try:
        for chunk, sb in ((2048, 1 << 30), (256, 1 << 17)):
            got, ref = c.decode(q, 0.0, chunk, sb)
            err = float(np.max(np.abs(got.astype(np.float64) - ref)))
            print(f"rising scores, decode chunk {chunk}: max|err| {err:.2e}", flush=True)
            assert np.isfinite(got).all() and err <= TOL
        q_len = np.array([600, 64, 777, 33], dtype=np.int32)
        q_rows = (0.3 * rng.standard_normal((int(q_len.sum()), Hq, D)) + 4.0 * u).astype(np.float32)
        for chunk, sb in ((2048, 1 << 30), (256, 1 << 18)):
            got, ref = c.prefill(q_rows, q_len, 0.0, chunk, sb)
            err = float(np.max(np.abs(got.astype(np.float64) - ref)))
            print(f"rising scores, prefill chunk {chunk}: max|err| {err:.2e}", flush=True)
            assert np.isfinite(got).all() and err <= TOL
    finally:
        c.close()
    # large logits through the scale: N(0,1) data, scale 2.2 -> logits ~ N(0, 25^2)
    K = [rng.standard_normal((n, Hkv, D)).astype(np.float32) for n in (300, 1030)]
    V = [rng.standard_normal((n, Hkv, D)).astype(np.float32) for n in (300, 1030)]
    q2 = rng.standard_normal((2, Hq, D)).astype(np.float32)
    c = Crafted(K, V, Hq, seed=7)
    try:
        got, ref = c.decode(q2, 2.2, 128, 1 << 16)
        err = float(np.max(np.abs(got.astype(np.float64) - ref)))
        print(f"logits ~ N(0, 25^2), decode: max|err| {err:.2e}", flush=True)
        assert np.isfinite(got).all() and err <= TOL
        q_len = np.array([120, 200], dtype=np.int32)
        q_rows = rng.standard_normal((320, Hq, D)).astype(np.float32)
        got, ref = c.prefill(q_rows, q_len, 2.2, 128, 1 << 17)
        err = float(np.max(np.abs(got.astype(np.float64) - ref)))
        print(f"logits ~ N(0, 25^2), prefill: max|err| {err:.2e}", flush=True)
        assert np.isfinite(got).all() and err <= TOL
    finally:
        c.close()


# ------------------------------------------------------------------ bad table entries, shared blocks
def test_bad_table_entry_is_flagged_and_other_sequences_are_untouched():
    from gpu_util import DeviceCase
    c = DeviceCase(synth.workload("llama8b_small"), seed=21)
    try:
        vkv, g = c.vkv, c.wl.geom
        c.plan(slice_bytes=1 << 20, chunk_tokens=256)
        q, q_t = c.q_dev(0)
        clean = c.attention(0, q_t)
        victim = int(np.argmax(c.st.ctx_len))
        bad = c.tables_t.clone()
        bad[victim, 1] = g.num_blocks + 5          # outside the pool
        bad[victim, 3] = -7                         # negative
        out = torch.full((c.wl.num_seqs, g.num_q_heads, g.head_dim), float("nan"), dtype=torch.float32, device="cuda:0")
        st, _ = vkv.kv_attn_run_layer(c.pool, 0, 0, q_t, bad, c.ws, out)
        assert st == vkv.VKV_OK
        with pytest.raises(vkv.VkvError) as e:
            vkv.kv_attn_check(c.pool, c.ws)
        assert e.value.code == vkv.VKV_E_STATE
        got = out.cpu().numpy()
        others = [s for s in range(c.wl.num_seqs) if s != victim]
        assert np.array_equal(got[others], clean[others])
        assert np.isfinite(got[victim]).all()       # the bad blocks were skipped, nothing wild was read
        # a new bind clears the flag
        vkv.kv_attn_bind(c.pool, c.ws)
        assert np.array_equal(c.attention(0, q_t), clean)
        # prefill: same tables, same verdict
        q_len = np.minimum(c.st.ctx_len, 100).astype(np.int32)
        total = int(q_len.sum())
        pq = synth.hash_bf16_bits(np.arange(total * g.num_q_heads * g.head_dim, dtype=np.int64), 5, 1)
        pq_t = torch.from_numpy(pq.reshape(total, g.num_q_heads, g.head_dim).view(np.int16)).cuda()
        info = vkv.kv_prefill_plan(c.pool, c.st.ctx_len, q_len, 1 << 20, 256)
        pws = torch.empty(info.workspace_bytes, dtype=torch.uint8, device="cuda:0")
        # a second pattern hits the first block of an item (the first of the sequence, and the first of its
        # second chunk), for which the kernel has nothing earlier to fall back on
        assert c.st.ctx_len[victim] > 17 * 16
        bad_first = c.tables_t.clone()
        bad_first[victim, 0] = -1
        bad_first[victim, 16] = g.num_blocks
        outs = []
        for tab in (c.tables_t, bad, bad_first):
            vkv.kv_prefill_bind(c.pool, pws)
            po = torch.full((total, g.num_q_heads, g.head_dim), float("nan"), dtype=torch.float32, device="cuda:0")
            st, _ = vkv.kv_prefill_run_layer(c.pool, 0, 0, pq_t, tab, pws, po)
            assert st == vkv.VKV_OK
            if tab is c.tables_t:
                vkv.kv_prefill_check(c.pool, pws)
            else:
                with pytest.raises(vkv.VkvError) as e:
                    vkv.kv_prefill_check(c.pool, pws)
                assert e.value.code == vkv.VKV_E_STATE
            outs.append(po.cpu().numpy())
        q_start = np.concatenate([[0], np.cumsum(q_len)])
        for other in outs[1:]:
            for s in others:
                assert np.array_equal(outs[0][q_start[s]:q_start[s + 1]], other[q_start[s]:q_start[s + 1]])
    finally:
        c.close()


def test_attention_over_blocks_shared_by_two_sequences():
    """Sequence 1 shares its first blocks with sequence 0 (a common prefix): both read the same blocks,
    decode and prefill agree with the oracle, and a reclamation that moves shared blocks rewrites both rows."""
    from gpu_util import DeviceCase, layout_of
    wl = synth.workload("llama8b_small", shared_prefix_blocks=9, ctx_dist=("uniform", 400, 1200))
    c = DeviceCase(wl, seed=31)
    try:
        vkv, g = c.vkv, wl.geom
        lay = layout_of(g)
        assert np.array_equal(c.st.tables[0, :9], c.st.tables[1, :9])
        c.plan(slice_bytes=1 << 19, chunk_tokens=128)
        q, q_t = c.q_dev(1)
        got = c.attention(1, q_t)
        ref = paged_decode_attention(c.pool_bits, lay, q, c.st.tables, c.st.ctx_len, 1)
        assert float(np.max(np.abs(got.astype(np.float64) - ref))) <= TOL
        # move everything out of the range that holds the most shared blocks
        bph = g.blocks_per_handle
        handles = c.st.tables[0, :9] // bph
        h = int(np.bincount(handles).argmax())
        vkv.kv_reclaim_range(c.pool, h * bph, (h + 1) * bph, c.tables_t, c.remap_t)
        tabs = c.tables_t.cpu().numpy()
        assert np.array_equal(tabs[0, :9], tabs[1, :9]) and not np.array_equal(tabs[0, :9], c.st.tables[0, :9])
        assert not ((tabs >= h * bph) & (tabs < (h + 1) * bph)).any()
        assert np.array_equal(c.attention(1, q_t), got)          # same bits after the move
    finally:
        c.close()
