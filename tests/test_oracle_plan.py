"""Pins for the attention plan oracle: exact cover, slice bound, maximality."""
import numpy as np
import pytest

from oracle.plan import attention_plan, balanced_attention_plan


@pytest.mark.parametrize("ctx,hkv,chunk,slice_bytes", [
    ([1], 1, 16, 1), ([16, 17, 255, 256, 257], 8, 64, 64 * 512 * 3),
    ([4096, 33, 512, 513, 8192], 2, 512, 1 << 20), ([100] * 7, 8, 128, 10 ** 9)])
def test_plan_covers_every_token_once_and_bounds_slices(ctx, hkv, chunk, slice_bytes):
    D, B = 128, 16
    work, starts = attention_plan(ctx, hkv, D, B, chunk, slice_bytes)
    seen = {}
    for s, h, fb, nt in work.tolist():
        assert 1 <= nt <= chunk and (fb * B) % chunk == 0
        for t in range(fb * B, fb * B + nt):
            assert (s, h, t) not in seen
            seen[(s, h, t)] = 1
    assert len(seen) == sum(ctx) * hkv
    assert all((s, h, t) in seen for s, n in enumerate(ctx) for h in range(hkv) for t in (0, n - 1))
    # launch order: sequence, then chunk, then head
    keys = [(s, fb, h) for s, h, fb, _ in work.tolist()]
    assert keys == sorted(keys)
    assert starts[0] == 0 and starts[-1] == len(work) and np.all(np.diff(starts) >= 1)
    nbytes = work[:, 3].astype(np.int64) * (2 * D * 2)
    for a, b in zip(starts[:-1], starts[1:]):
        tot = int(nbytes[a:b].sum())
        assert tot <= slice_bytes or b - a == 1
        if b < len(work):                       # maximal: the next item would not have fitted
            assert tot + int(nbytes[b]) > slice_bytes


def test_plan_rejects_bad_arguments():
    with pytest.raises(ValueError):
        attention_plan([5], 1, 64, 16, 24, 100)
    with pytest.raises(ValueError):
        attention_plan([5, -1], 1, 64, 16, 32, 100)


def test_absent_sequences_contribute_no_work():
    # a context length of 0 = a request that left the batch: the plan is that of the others, sequence ids kept
    w0, s0 = attention_plan([70, 0, 33], 2, 128, 16, 32, 10 ** 9)
    assert sorted(set(w0[:, 0].tolist())) == [0, 2]
    w1, _ = attention_plan([70, 33], 2, 128, 16, 32, 10 ** 9)
    w1 = w1.copy()
    w1[w1[:, 0] == 1, 0] = 2
    assert np.array_equal(w0, w1)
    wb, sb, qb = balanced_attention_plan([70, 0, 33], 2, 128, 16, 10 ** 9, 4)
    assert sorted(set(wb[:, 0].tolist())) == [0, 2] and int(wb[:, 3].sum()) == (70 + 33) * 2


# ------------------------------------------------------------------ equal shares
def test_balanced_plan_worked_by_hand():
    # two sequences of 40 and 100 tokens, 2 kv heads, units of 32 tokens:
    #   pair (0,0): units 32+8      stream positions 0-1
    #   pair (0,1): units 32+8      2-3
    #   pair (1,0): units 32+32+32+4   4-7
    #   pair (1,1): units 32+32+32+4   8-11        12 units in all, one slice
    # 3 queues: shares 0-3, 4-7, 8-11 = pairs (0,0)+(0,1) | (1,0) | (1,1)
    work, starts, queue = balanced_attention_plan([40, 100], 2, 128, 16, 10 ** 9, 3)
    assert work.tolist() == [[0, 0, 0, 40], [0, 1, 0, 40], [1, 0, 0, 100], [1, 1, 0, 100]]
    assert starts.tolist() == [0, 4] and queue.tolist() == [0, 0, 1, 2]
    # 5 queues: boundaries floor(j*12/5) = 0, 2, 4, 7, 9, 12
    #   q0 = (0,0) whole; q1 = (0,1) whole; q2 = units 0-2 of (1,0) = 96 tokens from block 0;
    #   q3 = unit 3 of (1,0) = 4 tokens from block 6, then unit 0 of (1,1) = 32 tokens;
    #   q4 = units 1-3 of (1,1) = 68 tokens from block 2
    work, starts, queue = balanced_attention_plan([40, 100], 2, 128, 16, 10 ** 9, 5)
    assert work.tolist() == [[0, 0, 0, 40], [0, 1, 0, 40], [1, 0, 0, 96], [1, 0, 6, 4], [1, 1, 0, 32], [1, 1, 2, 68]]
    assert queue.tolist() == [0, 1, 2, 3, 3, 4]
    # slices of 5 units (5 * 32 * 512 bytes): 0-4 | 5-9 | 10-11, 2 queues each:
    #   slice 0: units 0-1 | 2-4 -> (0,0) whole | (0,1) whole, (1,0) unit 0
    #   slice 1: units 5-6 | 7-9 -> (1,0) units 1-2 | (1,0) unit 3, (1,1) units 0-1
    #   slice 2: unit 10 | unit 11 -> (1,1) unit 2 | (1,1) unit 3
    work, starts, queue = balanced_attention_plan([40, 100], 2, 128, 16, 5 * 32 * 512, 2)
    assert work.tolist() == [[0, 0, 0, 40], [0, 1, 0, 40], [1, 0, 0, 32], [1, 0, 2, 64], [1, 0, 6, 4], [1, 1, 0, 64],
                             [1, 1, 4, 32], [1, 1, 6, 4]]
    assert starts.tolist() == [0, 3, 6, 8] and queue.tolist() == [0, 1, 1, 2, 3, 3, 4, 5]
    # an item never exceeds the bound: one pair of 100 tokens, one queue, at most 64 tokens per item
    work, _, queue = balanced_attention_plan([100], 1, 128, 16, 10 ** 9, 1, max_item_tokens=64)
    assert work.tolist() == [[0, 0, 0, 64], [0, 0, 4, 36]] and queue.tolist() == [0, 0]


@pytest.mark.parametrize("ctx,hkv,slice_bytes,slots", [
    ([1], 1, 1, 1), ([16, 17, 255, 256, 257], 8, 64 * 512 * 3, 7), ([4096, 33, 512, 513, 8192], 2, 1 << 20, 512),
    ([100] * 7, 8, 10 ** 9, 5), ([5000, 1, 2047, 2049], 1, 10 ** 9, 3), ([300, 0, 20], 4, 40000, 2)])
def test_balanced_plan_covers_every_token_once_in_equal_shares(ctx, hkv, slice_bytes, slots):
    D, B = 128, 16
    work, starts, queue = balanced_attention_plan(ctx, hkv, D, B, slice_bytes, slots)
    covered = []
    for s, h, fb, nt in work.tolist():
        assert 1 <= nt <= 2048 and (fb * B) % 32 == 0 and fb * B + nt <= ctx[s]
        covered.extend((s, h, t) for t in range(fb * B, fb * B + nt))
    assert covered == [(s, h, t) for s, n in enumerate(ctx) for h in range(hkv) for t in range(n)]   # once, in stream order
    assert starts[0] == 0 and starts[-1] == len(work) and np.all(np.diff(starts) >= 1)
    assert np.all(np.diff(queue) >= 0) and (len(queue) == 0 or queue[0] == 0)
    units = -(-work[:, 3] // 32)                 # an item starts on a unit boundary, so this counts its units
    unit_bytes = 32 * 2 * D * 2
    slice_units = max(1, slice_bytes // unit_bytes)
    for k, (a, b) in enumerate(zip(starts[:-1], starts[1:])):
        u = int(units[a:b].sum())
        assert u <= slice_units and (u == slice_units or b == len(work))          # full except the last
        assert int(work[a:b, 3].sum()) * 2 * D * 2 <= slice_bytes or slice_units == 1
        qs = queue[a:b]
        per_queue = [int(units[a:b][qs == q].sum()) for q in np.unique(qs)]
        assert len(per_queue) == min(slots, u)
        assert max(per_queue) - min(per_queue) <= 1
        if a > 0:
            assert queue[a] == queue[a - 1] + 1                                       # queues are numbered through


def test_prefill_plan_covers_every_query_token_pair_once():
    from oracle.plan import prefill_plan
    ctx, qlen, Hq, Hkv = [300, 77, 2100, 40], [300, 5, 130, 40], 8, 2      # G = 4 -> 32 positions per tile
    work, starts, tiles, tile_base = prefill_plan(ctx, qlen, Hq, Hkv, 128, 16, 256, 300000)
    assert tile_base[0] == 0 and tile_base[-1] == len(work) and len(tile_base) == len(tiles) + 1
    rows = 0
    seen = set()
    for k, (s, row0, pos0, n_pos) in enumerate(tiles.tolist()):
        assert 1 <= n_pos <= 32 and pos0 + n_pos <= ctx[s] and pos0 >= ctx[s] - qlen[s]
        items = work[tile_base[k]:tile_base[k + 1]]
        assert len(items) % Hkv == 0 and np.all(items[:, 0] == k)
        for h in range(Hkv):
            mine = items[items[:, 1] == h]
            covered = []
            for _, _, fb, nt in mine.tolist():
                assert 1 <= nt <= 256 and (fb * 16) % 256 == 0
                covered.extend(range(fb * 16, fb * 16 + nt))
            assert covered == list(range(pos0 + n_pos))          # exactly what the tile's last position sees
        for i in range(n_pos):
            assert (s, pos0 + i) not in seen
            seen.add((s, pos0 + i))
        rows += n_pos
    assert rows == sum(qlen) and seen == {(s, ctx[s] - qlen[s] + i) for s in range(4) for i in range(qlen[s])}
    # q rows are packed sequence after sequence, tile after tile
    assert tiles[:, 1].tolist() == np.concatenate([[0], np.cumsum(tiles[:, 3])[:-1]]).tolist()
    nbytes = work[:, 3].astype(np.int64) * 512
    for a, b in zip(starts[:-1], starts[1:]):
        assert int(nbytes[a:b].sum()) <= 300000 or b - a == 1
        if b < len(work):
            assert int(nbytes[a:b].sum()) + int(nbytes[b]) > 300000
