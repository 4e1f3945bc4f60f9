"""Selective handle choice (Algorithm 1), MIAD headroom and the cooldown gate: pins for the
oracle and parity of the library's host code with it."""
import itertools
import math

import numpy as np
import pytest

import synth
from oracle.policy import CooldownGate, Miad, handle_requests, selective_handles


# ------------------------------------------------------------------ Algorithm 1: oracle pins
def test_worked_example_by_hand():
    # handles:   0:{a}  1:{a,b}  2:{b,c}  3:{}   costs a=5 b=2 c=4
    reqs = [{0}, {0, 1}, {1, 2}, set()]
    cost = {0: 5, 1: 2, 2: 4}
    # k=1: the empty handle costs nothing
    assert selective_handles(1, reqs, cost) == ([3], set(), 0)
    # k=2: then handle 0 (5) ties... handle 0 costs 5, handle 1 costs 7, handle 2 costs 6 -> 0
    assert selective_handles(2, reqs, cost) == ([3, 0], {0}, 5)
    # k=3: a is gone, so handle 1 now costs only b=2, cheaper than handle 2 (6)
    assert selective_handles(3, reqs, cost) == ([3, 0, 1], {0, 1}, 7)
    # k=4: b is gone too, handle 2 costs c=4
    assert selective_handles(4, reqs, cost) == ([3, 0, 1, 2], {0, 1, 2}, 11)
    # ties go to the lowest index
    assert selective_handles(2, [{0}, {1}, {2}], {0: 3, 1: 3, 2: 3})[0] == [0, 1]
    with pytest.raises(ValueError):
        selective_handles(5, reqs, cost)


def test_every_step_is_the_argmin_of_the_marginal_cost():
    rng = np.random.default_rng(0)
    for _ in range(200):
        n_h, n_r = int(rng.integers(2, 9)), int(rng.integers(1, 8))
        reqs = [set(rng.choice(n_r, size=rng.integers(0, n_r + 1), replace=False).tolist()) for _ in range(n_h)]
        cost = {r: int(rng.integers(1, 50)) for r in range(n_r)}
        k = int(rng.integers(1, n_h + 1))
        chosen, evicted, total = selective_handles(k, reqs, cost)
        assert len(set(chosen)) == k
        gone, acc = set(), 0
        for i, h in enumerate(chosen):
            marg = {x: sum(cost[r] for r in reqs[x] - gone) for x in range(n_h) if x not in chosen[:i]}
            assert marg[h] == min(marg.values())
            assert h == min(x for x, c in marg.items() if c == marg[h])     # tie -> lowest index
            acc += marg[h]
            gone |= reqs[h]
        assert gone == evicted and acc == total
        # the total is the cost of the evicted set, each request counted once
        assert total == sum(cost[r] for r in evicted)
        if k == 1:     # one handle: greedy is optimal
            assert total == min(sum(cost[r] for r in reqs[x]) for x in range(n_h))


def test_greedy_never_worse_than_taking_the_top_handles_blindly():
    # "Reclaiming a handle blindly may preempt more requests than necessary": on random fragmented
    # pools the selective choice costs at most as much as the k highest handles for k = 1,
    # and in aggregate over many pools for larger k.
    worse = better = 0
    for seed in range(30):
        wl = synth.workload("tiny", occupancy=0.6)
        st = synth.build_state(wl, seed, materialize_pool=False)
        g = wl.geom
        reqs = handle_requests(st.tables, g.num_blocks, g.blocks_per_handle)
        cost = {r: int((st.tables[r] >= 0).sum()) * 16 for r in range(st.tables.shape[0])}
        for k in (1, 4, 8):
            _, ev, total = selective_handles(k, reqs, cost)
            blind = set().union(*reqs[-k:])
            blind_cost = sum(cost[r] for r in blind)
            if k == 1:
                assert total <= blind_cost
            better += total < blind_cost
            worse += total > blind_cost
    assert better > 5 * max(1, worse)


# ------------------------------------------------------------------ Algorithm 1: library parity
@pytest.fixture(scope="module")
def vkv():
    import paper_2604_07874_amd as v
    return v


@pytest.mark.parametrize("name,seed", [("tiny", 0), ("tiny", 5), ("llama8b_small", 1), ("stress_small", 2)])
def test_select_and_invalidate_match_the_oracle(vkv, name, seed):
    wl = synth.workload(name)
    st = synth.build_state(wl, seed, materialize_pool=False)
    g = wl.geom
    p = vkv.kv_pool_init(g.num_layers, g.num_q_heads, g.num_kv_heads, g.head_dim, g.num_blocks, g.blocks_per_handle)
    vkv.kv_pool_adopt(p, np.flatnonzero(st.live).astype(np.int32))
    n_rows = st.tables.shape[0]
    cost = np.array([int((st.tables[r] >= 0).sum()) * 16 for r in range(n_rows)], dtype=np.int64)
    cost[:wl.num_seqs] = st.ctx_len
    reqs = handle_requests(st.tables, g.num_blocks, g.blocks_per_handle)
    n_handles = g.num_blocks // g.blocks_per_handle
    for k in (0, 1, 3, n_handles // 2, n_handles):
        handles, ev, total = vkv.kv_select_handles(p, st.tables, cost, k)
        oh, oev, ototal = selective_handles(k, reqs, dict(enumerate(cost.tolist())))
        assert handles.tolist() == oh and ev.tolist() == sorted(oev) and total == ototal
    with pytest.raises(vkv.VkvError) as ei:
        vkv.kv_select_handles(p, st.tables, cost, n_handles + 1)
    assert ei.value.code == vkv.VKV_E_NOSPACE
    # hand three chosen handles over: the invalidated ids are exactly the table entries inside them
    handles, ev, _ = vkv.kv_select_handles(p, st.tables, cost, 3)
    live0, _ = vkv.kv_pool_state(p, g.num_blocks)
    if any(reqs[h] for h in handles):                                      # too small an output: refused whole
        with pytest.raises(vkv.VkvError) as ei:
            vkv.kv_invalidate_handles(p, handles, st.tables, cap=0)
        assert ei.value.code == vkv.VKV_E_NOSPACE
        live1, ranges1 = vkv.kv_pool_state(p, g.num_blocks)
        assert np.array_equal(live0, live1) and ranges1 == []
    rows, cols, blks = vkv.kv_invalidate_handles(p, handles, st.tables)
    bph = g.blocks_per_handle
    want = [(r, c, int(st.tables[r, c])) for r in range(n_rows) for c in range(st.tables.shape[1])
            if st.tables[r, c] >= 0 and st.tables[r, c] // bph in set(handles.tolist())]
    assert list(zip(rows.tolist(), cols.tolist(), blks.tolist())) == want
    assert sorted(set(rows.tolist())) == ev.tolist()
    live2, ranges2 = vkv.kv_pool_state(p, g.num_blocks)
    expect = st.live.copy()
    for h in handles:
        expect[h * bph:(h + 1) * bph] = 0
    assert np.array_equal(live2, expect)
    assert sorted(ranges2) == sorted((int(h) * bph, (int(h) + 1) * bph) for h in handles)
    # handed-over handles are no longer candidates, and cannot be handed over twice
    h2, _, _ = vkv.kv_select_handles(p, st.tables, cost, n_handles - 3)
    assert not set(h2.tolist()) & set(handles.tolist())
    with pytest.raises(vkv.VkvError) as ei:
        vkv.kv_invalidate_handles(p, handles[:1], st.tables)
    assert ei.value.code == vkv.VKV_E_BUSY
    vkv.kv_pool_return_range(p, int(handles[0]) * bph, (int(handles[0]) + 1) * bph)
    vkv.kv_pool_destroy(p)


def test_eviction_makes_room_for_a_relocation_that_did_not_fit(vkv):
    # 100 % occupancy: relocation out of the top range finds no room; evicting the cheapest
    # handles elsewhere (Algorithm 1) frees enough, at the price of the evicted requests.
    wl = synth.workload("tiny", occupancy=1.0)
    st = synth.build_state(wl, 3, materialize_pool=False)
    g = wl.geom
    p = vkv.kv_pool_init(g.num_layers, g.num_q_heads, g.num_kv_heads, g.head_dim, g.num_blocks, g.blocks_per_handle)
    vkv.kv_pool_adopt(p, np.flatnonzero(st.live).astype(np.int32))
    lo, hi = wl.reclaim_range
    with pytest.raises(vkv.VkvError) as ei:
        vkv.kv_reclaim_plan(p, lo, hi, g.num_blocks)
    assert ei.value.code == vkv.VKV_E_NOSPACE
    n_rows = st.tables.shape[0]
    cost = np.array([int((st.tables[r] >= 0).sum()) * 16 for r in range(n_rows)], dtype=np.int64)
    # the framework's answer: drop whole requests chosen by Algorithm 1 until the range fits
    tables = st.tables.copy()
    dropped = []
    for k in range(1, g.num_blocks // g.blocks_per_handle):
        _, ev, _ = vkv.kv_select_handles(p, tables, cost, k)
        for r in ev:
            if r not in dropped:
                ids = tables[r][tables[r] >= 0]
                vkv.kv_pool_free(p, ids)
                tables[r] = -1
                dropped.append(int(r))
        try:
            remap, stats = vkv.kv_reclaim_plan(p, lo, hi, g.num_blocks)
            break
        except vkv.VkvError as e:
            assert e.code == vkv.VKV_E_NOSPACE
    assert dropped and stats.blocks_moved == int(vkv.kv_pool_state(p, g.num_blocks)[0][lo:hi].sum())
    vkv.kv_pool_check_tables(p, tables)
    vkv.kv_pool_destroy(p)


@pytest.mark.parametrize("name,seed,k", [("tiny", 0, 3), ("tiny", 7, 10), ("llama8b_small", 1, 5), ("stress_small", 2, 4)])
def test_evict_handles_matches_the_oracle(vkv, name, seed, k):
    """kv_evict_handles on host tables (no device tables given) against the oracle's eviction, state for state."""
    from oracle import reclaim as R
    from oracle.policy import fifo_handles, handle_requests
    wl = synth.workload(name, shared_prefix_blocks=3 if name != "tiny" else 0)
    st = synth.build_state(wl, seed, materialize_pool=False)
    g = wl.geom
    p = vkv.kv_pool_init(g.num_layers, g.num_q_heads, g.num_kv_heads, g.head_dim, g.num_blocks, g.blocks_per_handle)
    vkv.kv_pool_adopt(p, np.flatnonzero(st.live).astype(np.int32))
    n_rows = st.tables.shape[0]
    cost = np.array([int((st.tables[r] >= 0).sum()) * 16 for r in range(n_rows)], dtype=np.int64)
    orc = R.ReclaimOracle(g.num_blocks, g.blocks_per_handle, st.live, st.tables, None)
    tables = st.tables.copy()
    # the comparison policy: the first k handles
    reqs = handle_requests(tables, g.num_blocks, g.blocks_per_handle)
    fh, fe, ft = fifo_handles(k, reqs, cost.tolist())
    ev, total = vkv.kv_handles_cost(p, tables, cost, fh)
    assert ev.tolist() == sorted(fe) and total == ft
    for round_ in range(2):                       # twice: the second time with handles already handed over
        status, handles, evicted, inv, total = orc.evict(k, cost.tolist())
        assert status == R.OK
        info, h, ev, (rows, cols, blks) = vkv.kv_evict_handles(p, k, tables, cost)
        assert h.tolist() == handles and ev.tolist() == evicted and info.total_cost == total
        assert list(zip(rows.tolist(), cols.tolist(), blks.tolist())) == inv
        assert np.array_equal(tables, orc.tables)
        live, ranges = vkv.kv_pool_state(p, g.num_blocks, max_ranges=256)
        assert np.array_equal(live, orc.live) and ranges == orc.released
        vkv.kv_pool_check_tables(p, tables)
    # too small an output: refused whole, the number needed is reported
    snap, state = tables.copy(), vkv.kv_pool_state(p, g.num_blocks, max_ranges=256)
    try:
        info, _, _, _ = vkv.kv_evict_handles(p, 2, tables, cost, cap=0)
        assert info.n_invalidated == 0              # the two cheapest handles left were named by nobody
    except vkv.VkvError as e:
        assert e.code == vkv.VKV_E_NOSPACE and np.array_equal(tables, snap)
        after = vkv.kv_pool_state(p, g.num_blocks, max_ranges=256)
        assert np.array_equal(after[0], state[0]) and after[1] == state[1]
    vkv.kv_pool_destroy(p)


def test_reclaim_or_evict_and_partial_return_on_the_host_side(vkv):
    """Relocation that does not fit turns into an eviction (the planning part, no device work), and a
    handed-over range can be given back handle by handle."""
    from oracle import reclaim as R
    wl = synth.workload("tiny", occupancy=1.0)
    st = synth.build_state(wl, 3, materialize_pool=False)
    g = wl.geom
    p = vkv.kv_pool_init(g.num_layers, g.num_q_heads, g.num_kv_heads, g.head_dim, g.num_blocks, g.blocks_per_handle)
    vkv.kv_pool_adopt(p, np.flatnonzero(st.live).astype(np.int32))
    lo, hi = wl.reclaim_range
    with pytest.raises(vkv.VkvError) as ei:
        vkv.kv_reclaim_plan(p, lo, hi, g.num_blocks)
    assert ei.value.code == vkv.VKV_E_NOSPACE
    cost = np.array([int((st.tables[r] >= 0).sum()) * 16 for r in range(st.tables.shape[0])], dtype=np.int64)
    orc = R.ReclaimOracle(g.num_blocks, g.blocks_per_handle, st.live, st.tables, None)
    k = (hi - lo) // g.blocks_per_handle
    status, mode, payload = orc.reclaim_or_evict(lo, hi, cost.tolist())
    assert (status, mode) == (R.OK, 1)
    tables = st.tables.copy()
    info, h, ev, _ = vkv.kv_evict_handles(p, k, tables, cost)
    assert h.tolist() == payload[0] and ev.tolist() == payload[1] and np.array_equal(tables, orc.tables)
    # the online tenant gives the handles back one at a time, from the middle of a merged picture too
    bph = g.blocks_per_handle
    first = int(h[0])
    assert orc.return_range(first * bph, (first + 1) * bph) == R.OK
    vkv.kv_pool_return_range(p, first * bph, (first + 1) * bph)
    live, ranges = vkv.kv_pool_state(p, g.num_blocks, max_ranges=256)
    assert ranges == orc.released and np.array_equal(live, orc.live)
    with pytest.raises(vkv.VkvError):
        vkv.kv_pool_return_range(p, first * bph, (first + 1) * bph)
    vkv.kv_pool_destroy(p)
    # partial return of one relocated range
    p = vkv.kv_pool_init(1, 8, 8, 64, 32, 4)
    orc = R.ReclaimOracle(32, 4, [0] * 32, [[-1]], None)
    vkv.kv_invalidate_handles(p, [2, 3, 4, 5], np.array([[-1]], dtype=np.int32))
    for lo_, hi_, ok in ((6, 10, False), (9, 12, False), (20, 24, True), (12, 16, True), (8, 12, True), (8, 12, False)):
        if ok:
            vkv.kv_pool_return_range(p, lo_, hi_)
        else:
            with pytest.raises(vkv.VkvError):
                vkv.kv_pool_return_range(p, lo_, hi_)
    assert vkv.kv_pool_state(p, 32)[1] == [(16, 20)]
    vkv.kv_pool_destroy(p)


# ------------------------------------------------------------------ MIAD
MIAD_KW = dict(h_init=4, h_min=2, h_max=64, alpha=1.5, pressure_frac=0.9, t_init=1.0, t_min=0.25, t_max=30.0,
               t_up=2.0, t_down=0.25, window_s=20.0, target_rate=0.1)


def test_miad_rules():
    m = Miad(**MIAD_KW)
    # no pressure: nothing happens before T has passed, then one handle is released per T
    assert m.observe(0.0, 0) == (4, 0, 0, 0, 1.0)
    assert m.observe(0.9, 0) == (4, 0, 0, 0, 1.0)
    h, grow, rel, ev, t = m.observe(1.0, 0)
    assert (h, grow, rel, ev) == (3, 0, 1, 0) and t == 0.75          # rate 0 <= target: T falls by t_down
    h, grow, rel, ev, t = m.observe(1.75, 0)
    assert (h, rel) == (2, 1) and t == 0.5
    assert m.observe(2.25, 0)[:3] == (2, 0, 0)                        # never below h_min
    # pressure at 90 % of H: multiplicative growth
    h, grow, rel, ev, t = m.observe(2.3, 2)                           # 2 >= 0.9*2
    assert (h, grow, rel, ev) == (3, 1, 0, 1)
    h, grow, rel, ev, t = m.observe(2.4, 3)
    assert (h, grow, ev) == (5, 2, 1)                                 # ceil(3*1.5)
    # two events in a 20 s window = 0.1/s: not above the target; a third one is
    t_before = t
    h, grow, rel, ev, t = m.observe(2.5, 5)
    assert ev == 1 and h == 8 and t == min(30.0, t_before * 2.0)
    # headroom never shrinks to or below the usage
    m2 = Miad(**MIAD_KW)
    m2.observe(0.0, 3)
    assert m2.observe(5.0, 3)[:3] == (4, 0, 0)


def test_miad_library_matches_oracle_on_random_traces(vkv):
    rng = np.random.default_rng(1)
    for trial in range(20):
        kw = dict(MIAD_KW, alpha=float(rng.choice([1.25, 1.5, 2.0])), target_rate=float(rng.choice([0.05, 0.2, 1.0])))
        m = vkv.kv_miad_init(**kw)
        o = Miad(**kw)
        now, used = 0.0, 0
        for _ in range(400):
            now += float(rng.exponential(0.3))
            used = max(0, min(60, used + int(rng.integers(-3, 4)) + (8 if rng.random() < 0.03 else 0)))
            if rng.random() < 0.05:
                used = 0
            assert vkv.kv_miad_observe(m, now, used) == o.observe(now, used)
        vkv.kv_miad_destroy(m)
    with pytest.raises(vkv.VkvError):
        vkv.kv_miad_init(**dict(MIAD_KW, alpha=1.0))


def test_miad_drives_the_event_rate_towards_the_target():
    # Bursty usage: with a low target the controller keeps more headroom (longer T) and sees
    # fewer pressure events than with a high target.
    def run(target):
        m = Miad(**dict(MIAD_KW, target_rate=target))
        rng = np.random.default_rng(2)
        events, now, hs = 0, 0.0, []
        for i in range(20000):
            now += 0.05
            used = 12 if (i // 200) % 5 == 0 else 1          # a burst every 50 s lasting 10 s
            h, _, _, ev, _ = m.observe(now, used)
            events += ev
            hs.append(h)
        return events, float(np.mean(hs))
    ev_low, h_low = run(0.01)
    ev_high, h_high = run(1.0)
    assert ev_low < ev_high and h_low > h_high


# ------------------------------------------------------------------ cooldown gate
def synthetic_online_trace(rng, n_requests, max_gap):
    """(time, kind, request) events: each request is a run of busy periods (decode iterations)
    separated by gaps <= max_gap; requests are separated by long idle times."""
    t, ev = 0.0, []
    for r in range(n_requests):
        t += float(rng.uniform(20 * max_gap, 60 * max_gap))
        for it in range(int(rng.integers(3, 40))):
            ev.append((t, "busy", r))
            t += float(rng.uniform(0.2, 1.0) * max_gap)
            ev.append((t, "idle", r))
            t += float(rng.uniform(0.05, 1.0) * max_gap)
    return ev


def drive(gate_busy, gate_idle, gate_poll, events, dt):
    """Feeds the trace and polls every dt; returns preemptions per request."""
    per_request = {}
    i, t = 0, 0.0
    end = events[-1][0] + 1.0
    while t < end:
        while i < len(events) and events[i][0] <= t:
            when, kind, r = events[i]
            if kind == "busy":
                if gate_busy(when, r):
                    per_request[r] = per_request.get(r, 0) + 1
            else:
                gate_idle(when)
            i += 1
        gate_poll(t)
        t += dt
    return per_request


def test_gate_at_most_one_preemption_per_request_and_parity(vkv):
    rng = np.random.default_rng(3)
    max_gap = 0.004
    events = synthetic_online_trace(rng, 40, max_gap)
    # the largest gap is known from instrumentation (here: given), as in the paper
    o = CooldownGate(max_gap)
    per_req = drive(o.online_busy, o.online_idle, o.poll, events, dt=max_gap / 7)
    assert per_req and max(per_req.values()) == 1 and len(per_req) == 40
    g = vkv.kv_gate_init(max_gap)
    per_req_lib = drive(lambda t, r: vkv.kv_gate_online_busy(g, t, r), lambda t: vkv.kv_gate_online_idle(g, t),
                        lambda t: vkv.kv_gate_poll(g, t), events, dt=max_gap / 7)
    assert per_req_lib == per_req
    gap, n = vkv.kv_gate_stats(g)
    assert n == o.preemptions == 40 and gap == o.g and gap <= max_gap
    vkv.kv_gate_destroy(g)
    # cold start with G = 0: the gate learns G from the first request's gaps and then holds
    o2 = CooldownGate(0.0)
    per_req2 = drive(o2.online_busy, o2.online_idle, o2.poll, events, dt=max_gap / 7)
    late = [per_req2.get(r, 0) for r in range(5, 40)]
    assert max(late) <= 2 and np.mean(late) < 1.2 and per_req2[0] > 1
    # without the cooldown (wake up at once when idle) every iteration would preempt
    iters = sum(1 for e in events if e[1] == "busy")
    assert iters > 10 * 40
