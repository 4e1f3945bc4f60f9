"""The stored expected values under tests/golden/ (hand-derived cases and the oracle's own record)."""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import synth
from oracle import reclaim as R
from oracle.attention import PoolLayout, paged_decode_attention
from oracle.plan import attention_plan, prefill_plan
from oracle.policy import selective_handles
from oracle.prefill import paged_prefill_attention

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def load(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return json.load(f)


def f32_to_bf16_bits(x):
    u = np.asarray(x, dtype=np.float32).view(np.uint32)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


# ------------------------------------------------------------------ Algorithm 1, worked by hand
def test_algorithm1_examples_oracle():
    for case in load("algorithm1_examples.json")["cases"]:
        reqs = [set(r) for r in case["reqs"]]
        cost = {int(k): v for k, v in case["cost"].items()}
        for e in case["expect"]:
            handles, evicted, total = selective_handles(e["k"], reqs, cost)
            assert handles == e["handles"], case["name"]
            assert sorted(evicted) == e["evicted"] and total == e["total"], case["name"]


def test_algorithm1_examples_library():
    import paper_2604_07874_amd as vkv
    if not os.path.exists(vkv.library_path()):
        from paper_2604_07874_amd import build
        build.build(verbose=False)
    for case in load("algorithm1_examples.json")["cases"]:
        n_h = len(case["reqs"])
        n_r = max([int(k) for k in case["cost"]]) + 1
        width = max(1, max(len(r) for r in case["reqs"]))
        # one table row per request; handle h = blocks [h*width, (h+1)*width); a request holds one
        # block of every handle that lists it
        tables = np.full((n_r, n_h), -1, dtype=np.int32)
        for h, rs in enumerate(case["reqs"]):
            for j, r in enumerate(rs):
                tables[r, h] = h * width + j
        pool = vkv.kv_pool_init(1, 8, 8, 64, n_h * width, width)
        live = np.unique(tables[tables >= 0]).astype(np.int32)
        if len(live):
            vkv.kv_pool_adopt(pool, live)
        cost = np.array([case["cost"][str(r)] for r in range(n_r)], dtype=np.int64)
        try:
            for e in case["expect"]:
                handles, evicted, total = vkv.kv_select_handles(pool, tables, cost, e["k"])
                assert list(handles) == e["handles"], case["name"]
                assert sorted(int(r) for r in evicted) == e["evicted"] and total == e["total"], case["name"]
        finally:
            vkv.kv_pool_destroy(pool)


# ------------------------------------------------------------------ relocation, worked by hand
def test_relocation_example_oracle_and_library():
    import paper_2604_07874_amd as vkv
    ex = load("relocation_example.json")
    nb, bph = ex["num_blocks"], ex["blocks_per_handle"]
    orc = R.ReclaimOracle(nb, bph, ex["live"], ex["tables"], None)
    pool = vkv.kv_pool_init(1, 8, 8, 64, nb, bph)
    vkv.kv_pool_adopt(pool, np.flatnonzero(np.array(ex["live"])).astype(np.int32))
    try:
        for step in ex["steps"]:
            if "return" in step:
                lo, hi = step["return"]
                assert orc.return_range(lo, hi) == R.OK
                # the library's bookkeeping of handed-over ranges changes only in kv_reclaim_range
                # (a device call); its planner is compared below on the states it can reach
                continue
            lo, hi = step["reclaim"]
            status, src, dst, remap = orc.reclaim(lo, hi)
            assert status == step["status"], step["derivation"]
            moves = [] if src is None else [[int(a), int(b)] for a, b in zip(src, dst)]
            assert moves == step["moves"], step["derivation"]
            assert orc.tables.tolist() == step["tables_after"] and orc.live.tolist() == step["live_after"]
        # the library's host planner on the first step (no range handed over yet)
        first = ex["steps"][0]
        remap, stats = vkv.kv_reclaim_plan(pool, first["reclaim"][0], first["reclaim"][1], nb)
        got = [[int(b), int(remap[b])] for b in range(nb) if remap[b] != b]
        assert got == first["moves"] and stats.blocks_moved == len(first["moves"])
    finally:
        vkv.kv_pool_destroy(pool)


# ------------------------------------------------------------------ attention, exact rationals
def build_pool(fix):
    g = fix["geometry"]
    lay = PoolLayout(g["num_layers"], g["num_kv_heads"], g["head_dim"], g["block_tokens"])
    pool = np.full(g["num_blocks"] * lay.block_elems, synth.BF16_NAN_BITS, dtype=np.uint16)
    for blk, kv, head, slot, vals in fix["pool_entries"]:
        o = lay.vec_offset(blk, 0, kv, head, slot)
        pool[o:o + g["head_dim"]] = f32_to_bf16_bits(vals)
    return lay, pool


def scale_of(name):
    return {"ln2": math.log(2.0), "ln3": math.log(3.0)}[name]


def test_attention_exact_cases_decode():
    fix = load("attention_exact_cases.json")
    lay, pool = build_pool(fix)
    tables = np.array(fix["tables"], dtype=np.int32)
    ctx = np.array(fix["ctx_len"], dtype=np.int32)
    for case in fix["decode"]:
        q = f32_to_bf16_bits(np.array(case["q"], dtype=np.float32))
        out = paged_decode_attention(pool, lay, q, tables, ctx, 0, scale=scale_of(case["scale"]))
        want = np.array([[[float(Fraction(x)) for x in head] for head in seq] for seq in case["expect"]])
        assert np.allclose(out, want, rtol=0, atol=1e-14), case["name"]


def test_attention_exact_cases_prefill():
    fix = load("attention_exact_cases.json")
    lay, pool = build_pool(fix)
    tables = np.array(fix["tables"], dtype=np.int32)
    ctx = np.array(fix["ctx_len"], dtype=np.int32)
    for case in fix["prefill"]:
        q = f32_to_bf16_bits(np.array(case["q_seq0"], dtype=np.float32))
        q_len = np.array(case["q_len"], dtype=np.int32)
        out = paged_prefill_attention(pool, lay, q, np.array([0, q_len[0]]), q_len, tables, ctx, 0,
                                      scale=scale_of(case["scale"]), seqs=[0])
        want = np.array([[float(Fraction(x)) for x in row] for row in case["expect_seq0"]])
        for head in range(q.shape[1]):
            assert np.allclose(out[:, head], want, rtol=0, atol=1e-14), case["name"]


# ------------------------------------------------------------------ the oracle's own record
def test_oracle_output_has_not_drifted():
    rec = load("oracle_tiny_seed0.json")
    wl = synth.workload("tiny")
    g = wl.geom
    st = synth.build_state(wl, seed=0)
    assert [int(x) for x in st.ctx_len] == rec["ctx_len"]
    lay = PoolLayout(g.num_layers, g.num_kv_heads, g.head_dim, g.block_tokens)
    out = paged_decode_attention(st.pool_bits, lay, synth.query_bits(wl, 0, 0), st.tables, st.ctx_len, 0)
    for smp in rec["decode_samples"]:
        assert out[smp["seq"], smp["head"], smp["d"]] == pytest.approx(float(smp["value"]), rel=0, abs=1e-13)
    q_len = np.minimum(st.ctx_len, 5).astype(np.int32)
    q_start = np.concatenate([[0], np.cumsum(q_len)[:-1]]).astype(np.int64)
    total_q = int(q_len.sum())
    assert total_q == rec["prefill_rows"]
    pq = synth.hash_bf16_bits(np.arange(total_q * g.num_q_heads * g.head_dim, dtype=np.int64), 0, 7).reshape(
        total_q, g.num_q_heads, g.head_dim)
    pout = paged_prefill_attention(st.pool_bits, lay, pq, q_start, q_len, st.tables, st.ctx_len, 0)
    for smp in rec["prefill_samples"]:
        assert pout[smp["row"], smp["head"], smp["d"]] == pytest.approx(float(smp["value"]), rel=0, abs=1e-13)
    import hashlib

    def digest(a):
        return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()
    work, starts = attention_plan(st.ctx_len, g.num_kv_heads, g.head_dim, g.block_tokens, 64, 100000)
    ap = rec["attention_plan"]
    assert (len(work), len(starts) - 1, digest(np.asarray(work, dtype=np.int32))) == (ap["n_items"], ap["n_slices"], ap["work_sha256"])
    pwork, _, ptiles, _ = prefill_plan(st.ctx_len, q_len, g.num_q_heads, g.num_kv_heads, g.head_dim, g.block_tokens, 64, 100000)
    pp = rec["prefill_plan"]
    assert (len(pwork), len(ptiles), digest(np.asarray(pwork, dtype=np.int32))) == (pp["n_items"], pp["n_tiles"], pp["work_sha256"])
    lo, hi = rec["reclaim"]["range"]
    orc = R.ReclaimOracle(g.num_blocks, g.blocks_per_handle, st.live, st.tables, None)
    status, src, dst, _ = orc.reclaim(lo, hi)
    assert status == rec["reclaim"]["status"]
    assert [[int(a), int(b)] for a, b in zip(src, dst)] == rec["reclaim"]["moves"]
    assert digest(orc.tables.astype(np.int32)) == rec["reclaim"]["tables_sha256"]
    assert digest(orc.live.astype(np.uint8)) == rec["reclaim"]["live_sha256"]


# ------------------------------------------------------------------ MIAD and cooldown gate, stepped by hand
def _library():
    import paper_2604_07874_amd as vkv
    if not os.path.exists(vkv.library_path()):
        from paper_2604_07874_amd import build
        build.build(verbose=False)
    return vkv


def test_miad_traces_oracle():
    from oracle.policy import Miad
    traces = load("miad_traces.json")["traces"]
    assert len(traces) >= 2
    for tr in traces:
        assert len(tr["rows"]) >= 12 and len(tr["rows"]) == len(tr["why"])
        m = Miad(**tr["config"])
        for i, (now, used, h, grow, rel, ev, t) in enumerate(tr["rows"]):
            assert m.observe(now, used) == (h, grow, rel, ev, t), (tr["name"], i, tr["why"][i])


def test_miad_traces_library():
    vkv = _library()
    for tr in load("miad_traces.json")["traces"]:
        m = vkv.kv_miad_init(**tr["config"])
        try:
            for i, (now, used, h, grow, rel, ev, t) in enumerate(tr["rows"]):
                assert vkv.kv_miad_observe(m, now, used) == (h, grow, rel, ev, t), (tr["name"], i, tr["why"][i])
        finally:
            vkv.kv_miad_destroy(m)


def _run_gate(busy, idle, poll, steps, why, name):
    for i, (op, now, req, want) in enumerate(steps):
        if op == "busy":
            got = busy(now, req)
        elif op == "idle":
            idle(now)
            got = 0
        else:
            got = poll(now)
        assert got == want, (name, i, why[i])


def test_cooldown_traces_oracle():
    from oracle.policy import CooldownGate
    traces = load("cooldown_traces.json")["traces"]
    assert len(traces) >= 2
    for tr in traces:
        assert len(tr["steps"]) == len(tr["why"])
        g = CooldownGate(tr["initial_gap_s"])
        _run_gate(g.online_busy, g.online_idle, g.poll, tr["steps"], tr["why"], tr["name"])
        assert g.g == tr["final"]["max_gap_s"] and g.preemptions == tr["final"]["preemptions"]


def test_cooldown_traces_library():
    vkv = _library()
    for tr in load("cooldown_traces.json")["traces"]:
        g = vkv.kv_gate_init(tr["initial_gap_s"])
        try:
            _run_gate(lambda t, r: vkv.kv_gate_online_busy(g, t, r), lambda t: vkv.kv_gate_online_idle(g, t),
                      lambda t: vkv.kv_gate_poll(g, t), tr["steps"], tr["why"], tr["name"])
            assert vkv.kv_gate_stats(g) == (tr["final"]["max_gap_s"], tr["final"]["preemptions"])
        finally:
            vkv.kv_gate_destroy(g)


# ------------------------------------------------------------------ eviction by Algorithm 1, worked by hand
def _eviction_oracle(ex, case):
    return R.ReclaimOracle(ex["num_blocks"], ex["blocks_per_handle"], case["live"], case["tables"], None)


def test_eviction_examples_oracle():
    from oracle.policy import fifo_handles, handle_requests
    ex = load("eviction_examples.json")
    for case in ex["cases"]:
        orc = _eviction_oracle(ex, case)
        reqs = handle_requests(orc.tables, orc.nb, orc.bph)
        fh, fe, ft = fifo_handles(case["k"], reqs, case["cost"])
        assert (fh, sorted(fe), ft) == (case["fifo"]["handles"], case["fifo"]["evicted"], case["fifo"]["total"])
        st, handles, evicted, inv, total = orc.evict(case["k"], case["cost"])
        assert st == case["status"] and handles == case["handles"] and evicted == case["evicted"], case["name"]
        assert total == case["total"] and [list(x) for x in inv] == case["invalidated"], case["name"]
        assert orc.tables.tolist() == case["tables_after"] and orc.live.tolist() == case["live_after"], case["name"]
        assert [list(r) for r in orc.released] == case["released_after"], case["name"]
        assert total <= ft
    roe = ex["reclaim_or_evict"]
    orc = _eviction_oracle(ex, roe)
    st, mode, payload = orc.reclaim_or_evict(*roe["range"], roe["cost"])
    assert (st, mode) == (R.OK, roe["mode"]) and payload[0] == roe["handles"] and payload[1] == roe["evicted"]
    assert orc.live.tolist() == roe["live_after"]
    nxt = roe["then_relocation_fits"]
    st, mode, payload = orc.reclaim_or_evict(*nxt["range"], roe["cost"])
    assert (st, mode) == (R.OK, nxt["mode"])
    assert [[int(a), int(b)] for a, b in zip(payload[0], payload[1])] == nxt["moves"]


def test_eviction_examples_library():
    vkv = _library()
    ex = load("eviction_examples.json")
    nb, bph = ex["num_blocks"], ex["blocks_per_handle"]

    def make(case):
        p = vkv.kv_pool_init(1, 8, 8, 64, nb, bph)
        vkv.kv_pool_adopt(p, np.flatnonzero(np.array(case["live"])).astype(np.int32))
        return p, np.array(case["tables"], dtype=np.int32), np.array(case["cost"], dtype=np.int64)

    for case in ex["cases"]:
        p, tables, cost = make(case)
        try:
            fifo = [h for h in range(nb // bph)][:case["k"]]
            ev, total = vkv.kv_handles_cost(p, tables, cost, fifo)
            assert (ev.tolist(), total) == (case["fifo"]["evicted"], case["fifo"]["total"])
            info, handles, evicted, (rows, cols, blks) = vkv.kv_evict_handles(p, case["k"], tables, cost)
            assert (info.mode, info.n_handles, info.total_cost) == (1, case["k"], case["total"]), case["name"]
            assert handles.tolist() == case["handles"] and evicted.tolist() == case["evicted"], case["name"]
            assert [list(x) for x in zip(rows.tolist(), cols.tolist(), blks.tolist())] == case["invalidated"], case["name"]
            assert tables.tolist() == case["tables_after"], case["name"]
            live, ranges = vkv.kv_pool_state(p, nb)
            assert live.tolist() == case["live_after"] and [list(r) for r in ranges] == case["released_after"], case["name"]
        finally:
            vkv.kv_pool_destroy(p)
