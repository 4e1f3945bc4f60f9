"""Pins for the attention plan oracle: exact cover, slice bound, maximality."""
import numpy as np
import pytest

from oracle.plan import attention_plan


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
