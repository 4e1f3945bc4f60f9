"""Pins for the reclamation oracle: a dictionary-based simulator and conservation invariants."""
import numpy as np
import pytest

import synth
from oracle import reclaim as R
from oracle.attention import PoolLayout, gather_contiguous, paged_decode_attention


def layout_of(g):
    return PoolLayout(g.num_layers, g.num_kv_heads, g.head_dim, g.block_tokens)


def dict_simulator(nb, bph, live_set, tables, contents, released, lo, hi):
    """Independent restatement with sets and dicts; returns new (live, tables, contents, moves)."""
    assert lo % bph == 0 and hi % bph == 0 and 0 <= lo < hi <= nb
    inside = sorted(b for b in live_set if lo <= b < hi)
    banned = set(range(lo, hi))
    for rlo, rhi in released:
        banned |= set(range(rlo, rhi))
    free = sorted(set(range(nb)) - set(live_set) - banned)
    if len(free) < len(inside):
        return None
    moves = dict(zip(inside, free))
    new_live = (set(live_set) - set(inside)) | set(moves.values())
    new_contents = dict(contents)
    for s, d in moves.items():
        new_contents[d] = contents[s]
    new_tables = [[moves.get(e, e) if e >= 0 else e for e in row] for row in tables]
    return new_live, new_tables, new_contents, moves


@pytest.fixture()
def tiny_state():
    wl = synth.workload("tiny", shared_prefix_blocks=1, ctx_dist=("uniform", 40, 256))
    st = synth.build_state(wl, seed=1)
    g = wl.geom
    pool = st.pool_bits.reshape(g.num_blocks, g.block_elems).copy()
    return wl, st, pool


def make_oracle(wl, st, pool):
    g = wl.geom
    return R.ReclaimOracle(g.num_blocks, g.blocks_per_handle, st.live, st.tables, pool)


def test_matches_dictionary_simulator(tiny_state):
    wl, st, pool = tiny_state
    g = wl.geom
    orc = make_oracle(wl, st, pool)
    live = set(np.flatnonzero(st.live).tolist())
    tables = st.tables.tolist()
    contents = {b: pool[b].tobytes() for b in range(g.num_blocks)}
    released = []
    for lo, hi in [(192, 256), (0, 16), (96, 104)]:
        status, src, dst, remap = orc.reclaim(lo, hi)
        sim = dict_simulator(g.num_blocks, g.blocks_per_handle, live, tables, contents, released, lo, hi)
        assert status == R.OK and sim is not None
        live, tables, contents, moves = sim
        released.append((lo, hi))
        assert dict(zip(src.tolist(), dst.tolist())) == moves
        assert set(np.flatnonzero(orc.live).tolist()) == live
        assert orc.tables.tolist() == tables
        for b in live:
            assert orc.pool[b].tobytes() == contents[b]
        assert all(remap[b] == moves.get(b, b) for b in range(g.num_blocks))


def test_invariants_after_reclaim(tiny_state):
    wl, st, pool = tiny_state
    g = wl.geom
    lay = layout_of(g)
    lo, hi = wl.reclaim_range
    before_pool = pool.copy()
    q = synth.query_bits(wl, 1, 0)
    out_before = paged_decode_attention(pool.reshape(-1), lay, q, st.tables, st.ctx_len, 0)
    gathered_before = [gather_contiguous(pool.reshape(-1), lay, st.tables[s], int(st.ctx_len[s]), 0)
                       for s in range(wl.num_seqs)]
    orc = make_oracle(wl, st, pool)
    status, src, dst, remap = orc.reclaim(lo, hi)
    assert status == R.OK and len(src) == st.live[lo:hi].sum() > 0
    assert orc.live[lo:hi].sum() == 0                                   # range holds nothing live
    assert orc.live.sum() == st.live.sum()                              # live count conserved
    assert np.all((src >= lo) & (src < hi)) and np.all(dst < lo)
    assert np.all(np.diff(src) > 0) and np.all(np.diff(dst) > 0)        # ascending pairing
    assert np.all(st.live[dst] == 0)
    # every free block below the last destination was used: lowest free ids first
    assert set(dst.tolist()) == set(np.flatnonzero(st.live[:lo] == 0)[:len(src)].tolist())
    # untouched blocks keep their bytes
    untouched = np.setdiff1d(np.arange(lo), dst)
    assert np.array_equal(orc.pool[untouched], before_pool[untouched])
    # every sequence gathers the same bytes through the rewritten table
    for s in range(wl.num_seqs):
        Kb, Vb = gather_contiguous(orc.pool.reshape(-1), lay, orc.tables[s], int(st.ctx_len[s]), 0)
        assert np.array_equal(Kb, gathered_before[s][0]) and np.array_equal(Vb, gathered_before[s][1])
    used = orc.tables[orc.tables >= 0]
    assert np.all(used < lo) and np.all(orc.live[used] == 1)
    # the shared prefix block still is shared
    assert orc.tables[0, 0] == orc.tables[1, 0]
    # poisoning the released range leaves attention unchanged (bitwise)
    orc.pool[lo:hi] = synth.BF16_NAN_BITS
    out_after = paged_decode_attention(orc.pool.reshape(-1), lay, q, orc.tables, st.ctx_len, 0)
    assert np.array_equal(out_before, out_after)


def test_error_paths_leave_state_untouched(tiny_state):
    wl, st, pool = tiny_state
    orc = make_oracle(wl, st, pool)
    snap = (orc.live.copy(), orc.tables.copy(), orc.pool.copy())

    def unchanged():
        return (np.array_equal(orc.live, snap[0]) and np.array_equal(orc.tables, snap[1])
                and np.array_equal(orc.pool, snap[2]) and orc.released == [])

    for lo, hi in [(-8, 8), (8, 8), (16, 8), (4, 16), (0, 12), (248, 264)]:
        assert orc.reclaim(lo, hi)[0] == R.E_INVAL and unchanged()
    # 128 live blocks cannot fit into what is left outside a 200-block range
    assert orc.reclaim(0, 200)[0] == R.E_NOSPACE and unchanged()


def test_repeat_return_and_overlap(tiny_state):
    wl, st, pool = tiny_state
    orc = make_oracle(wl, st, pool)
    lo, hi = wl.reclaim_range
    assert orc.reclaim(lo, hi)[0] == R.OK
    assert orc.reclaim(lo, hi)[0] == R.E_BUSY                 # already handed over
    assert orc.reclaim(lo - 8, lo + 8)[0] == R.E_BUSY
    # a second, disjoint range never uses the first one as destination
    status, src, dst, _ = orc.reclaim(lo - 64, lo)
    assert status == R.OK and np.all(dst < lo - 64)
    assert orc.return_range(lo, hi) == R.OK
    assert orc.return_range(lo, hi) == R.E_INVAL
    # after the return the range is free space again: reclaiming it moves nothing
    status, src, dst, _ = orc.reclaim(lo, hi)
    assert status == R.OK and len(src) == 0
    assert orc.return_range(lo, hi) == R.OK
    # and it can serve as destination for a later reclaim of a low range
    status, src, dst, _ = orc.reclaim(0, 64)
    assert status == R.OK and len(src) > 0 and np.all(dst >= 64)


def test_unreferenced_live_blocks_are_moved_too():
    live = np.zeros(32, dtype=np.uint8)
    live[[3, 17, 30, 31]] = 1
    tables = np.array([[30, 3, -1]], dtype=np.int32)        # 17 and 31 are live but unreferenced
    pool = np.arange(32 * 4, dtype=np.uint16).reshape(32, 4)
    orc = R.ReclaimOracle(32, 8, live, tables, pool)
    status, src, dst, remap = orc.reclaim(24, 32)
    assert status == R.OK and src.tolist() == [30, 31] and dst.tolist() == [0, 1]
    assert orc.tables.tolist() == [[0, 3, -1]]
    assert orc.pool[1].tolist() == [124, 125, 126, 127]


# ------------------------------------------------------------------ eviction (the paper's own hand-over)
@pytest.mark.parametrize("seed", range(6))
def test_eviction_invariants_on_random_pools(seed):
    import synth
    from oracle.policy import handle_requests
    wl = synth.workload("tiny", occupancy=0.9, shared_prefix_blocks=2 if seed % 2 else 0)
    st = synth.build_state(wl, seed, materialize_pool=False)
    g = wl.geom
    n_rows = st.tables.shape[0]
    cost = [int((st.tables[r] >= 0).sum()) * 16 for r in range(n_rows)]
    orc = R.ReclaimOracle(g.num_blocks, g.blocks_per_handle, st.live, st.tables, None)
    before_tables, before_live = orc.tables.copy(), orc.live.copy()
    reqs = handle_requests(before_tables, g.num_blocks, g.blocks_per_handle)
    k = 3
    status, handles, evicted, inv, total = orc.evict(k, cost)
    assert status == R.OK and len(set(handles)) == k
    bph = g.blocks_per_handle
    chosen = set(handles)
    # the evicted requests are exactly those with a block in a chosen handle, and their cost is the total
    assert set(evicted) == set().union(*[reqs[h] for h in handles])
    assert total == sum(cost[r] for r in evicted)
    # invalidated entries = brute force over the old tables
    want = [(r, c, int(before_tables[r, c])) for r in range(n_rows) for c in range(before_tables.shape[1])
            if before_tables[r, c] >= 0 and int(before_tables[r, c]) // bph in chosen]
    assert inv == want
    # survivors keep their rows, evicted rows are empty, nobody names a chosen handle any more
    for r in range(n_rows):
        if r in evicted:
            assert (orc.tables[r] == -1).all()
        else:
            assert np.array_equal(orc.tables[r], before_tables[r])
    used = orc.tables[orc.tables >= 0]
    assert not np.isin(used // bph, list(chosen)).any()
    # every block a survivor names is still live; chosen handles are dead and handed over
    assert orc.live[used].all()
    for h in handles:
        assert not orc.live[h * bph:(h + 1) * bph].any()
    assert sorted(orc.released) == sorted((h * bph, (h + 1) * bph) for h in handles)
    # nothing that was dead came alive, and blocks outside evicted rows and chosen handles are untouched
    assert not (orc.live & ~before_live.astype(bool)).any()
    gone = set(np.flatnonzero(before_live.astype(bool) & ~orc.live.astype(bool)).tolist())
    ev_blocks = {int(e) for r in evicted for e in before_tables[r] if e >= 0}
    handle_blocks = {b for h in handles for b in range(h * bph, (h + 1) * bph)}
    assert gone <= ev_blocks | handle_blocks
    # handed-over handles are no candidates any more; asking for more handles than are left fails whole
    n_handles = g.num_blocks // bph
    snap = (orc.tables.copy(), orc.live.copy(), list(orc.released))
    assert orc.evict(n_handles - k + 1, cost)[0] == R.E_NOSPACE
    assert np.array_equal(orc.tables, snap[0]) and np.array_equal(orc.live, snap[1]) and orc.released == snap[2]


def test_selective_choice_costs_no_more_than_fifo():
    """Section 7.2 compares Algorithm 1 with evicting in first-in-first-out order: for one handle the
    greedy choice is the minimum, and over many fragmented pools it is cheaper in aggregate."""
    import synth
    from oracle.policy import fifo_handles, handle_requests, selective_handles
    better = worse = 0
    for seed in range(40):
        wl = synth.workload("tiny", occupancy=0.7)
        st = synth.build_state(wl, seed, materialize_pool=False)
        g = wl.geom
        reqs = handle_requests(st.tables, g.num_blocks, g.blocks_per_handle)
        cost = {r: int((st.tables[r] >= 0).sum()) * 16 for r in range(st.tables.shape[0])}
        for k in (1, 2, 4, 8):
            _, _, sel = selective_handles(k, reqs, cost)
            _, _, fifo = fifo_handles(k, reqs, cost)
            if k == 1:
                assert sel <= fifo
            better += sel < fifo
            worse += sel > fifo
    assert better > 5 * max(1, worse)


def test_return_of_part_of_a_range():
    orc = R.ReclaimOracle(32, 4, [0] * 32, [[-1]], None)
    assert orc.reclaim(8, 24)[0] == R.OK
    assert orc.return_range(6, 10) == R.E_INVAL        # not inside one handed-over range
    assert orc.return_range(9, 12) == R.E_INVAL        # not handle-aligned
    assert orc.return_range(20, 24) == R.OK and orc.released == [(8, 20)]       # from the top
    assert orc.return_range(12, 16) == R.OK and orc.released == [(8, 12), (16, 20)]   # from the middle: a split
    assert orc.return_range(8, 12) == R.OK and orc.released == [(16, 20)]
    assert orc.return_range(8, 12) == R.E_INVAL        # already back
    assert orc.reclaim(16, 20)[0] == R.E_BUSY
    assert orc.return_range(16, 20) == R.OK and orc.released == []
