"""Relocation of live KV blocks out of a reclaimed range + block-table rewrite (test oracle).

Problem statement followed (Section 2.3, Challenge 2; Section 5, "Sub-layer
memory reclamation"): when the online tenant needs memory, a set of the offline
tenant's equal-size handles must be handed over promptly, without the offline
job touching reclaimed memory afterwards and without killing it.  The paper
makes the handles harmless by remapping them and lets the framework recompute
the lost KV; this library keeps the KV instead: every live block inside the
range is copied to a free block outside it and every block-table entry that
named it is rewritten, so the offline job reads the same bytes as before.

Rule that makes the result unique (a choice of this library): the i-th live
block of the range in ascending id order moves to the i-th free block, in
ascending id order, that lies outside the range and outside every range
already handed over.

State: pool bytes, live[NB], block tables, list of released ranges.
"""
from __future__ import annotations

import numpy as np

OK, E_INVAL, E_NOSPACE, E_BUSY = 0, -1, -2, -3


class ReclaimOracle:
    def __init__(self, num_blocks: int, blocks_per_handle: int, live, tables,
                 pool_blocks=None):
        """pool_blocks: optional uint16 [NB, block_elems] array, modified in place."""
        self.nb = int(num_blocks)
        self.bph = int(blocks_per_handle)
        self.live = np.array(live, dtype=np.uint8).copy()
        self.tables = np.array(tables, dtype=np.int32).copy()
        self.pool = pool_blocks
        self.released = []  # list of (lo, hi)

    # ------------------------------------------------------------------
    def _in_released(self, b: int) -> bool:
        return any(lo <= b < hi for lo, hi in self.released)

    def check_range(self, lo: int, hi: int) -> int:
        if lo < 0 or hi > self.nb or lo >= hi or lo % self.bph or hi % self.bph:
            return E_INVAL
        if any(lo < rhi and rlo < hi for rlo, rhi in self.released):
            return E_BUSY
        return OK

    def reclaim(self, lo: int, hi: int):
        """Returns (status, src, dst, remap).  On failure the state is untouched."""
        st = self.check_range(lo, hi)
        if st != OK:
            return st, None, None, None
        src = [b for b in range(lo, hi) if self.live[b]]
        dst = []
        for b in range(self.nb):
            if len(dst) == len(src):
                break
            if lo <= b < hi or self.live[b] or self._in_released(b):
                continue
            dst.append(b)
        if len(dst) < len(src):
            return E_NOSPACE, None, None, None
        remap = np.arange(self.nb, dtype=np.int32)
        for s, d in zip(src, dst):
            if self.pool is not None:
                self.pool[d] = self.pool[s]
            self.live[d] = 1
            self.live[s] = 0
            remap[s] = d
        used = self.tables >= 0
        self.tables[used] = remap[self.tables[used]]
        self.released.append((lo, hi))
        return OK, np.asarray(src, dtype=np.int32), np.asarray(dst, dtype=np.int32), remap

    def return_range(self, lo: int, hi: int) -> int:
        """The online tenant gives back handles it holds: [lo, hi) must be handle-aligned and lie inside
        one released range, which shrinks or splits accordingly (the dynamic reservation of Section 5
        releases one handle at a time); the returned blocks are free again."""
        if lo < 0 or hi > self.nb or lo >= hi or lo % self.bph or hi % self.bph:
            return E_INVAL
        for i, (rlo, rhi) in enumerate(self.released):
            if rlo <= lo and hi <= rhi:
                rest = [r for r in ((rlo, lo), (hi, rhi)) if r[0] < r[1]]
                self.released[i:i + 1] = rest
                return OK
        return E_INVAL

    # ------------------------------------------------------------------
    def evict(self, k: int, cost):
        """The paper's own hand-over (Section 5, "Sub-layer memory reclamation" and "Selective handle
        reclamation"): k handles chosen by Algorithm 1 are handed over without saving their contents;
        every request with a block in one of them is evicted whole (it goes back to the waiting state
        and is recomputed later), and the table entries that named blocks of the chosen handles are
        reported per request: the invalidated ids.

        cost[r] = Cost(r) for table row r.  Candidates are the handles outside every released range.
        Returns (status, handles in pick order, evicted rows ascending, invalidated [(row, col, block)]
        in row-major order, total cost).  Afterwards: the evicted rows are empty; every block of the
        chosen handles is dead; a block of an evicted row elsewhere is dead unless a surviving row
        still names it; each chosen handle is a released range.  On failure nothing has changed."""
        from .policy import handle_requests, selective_handles
        n_handles = self.nb // self.bph
        cand = [h for h in range(n_handles) if not self._in_released(h * self.bph)]
        if k < 0:
            return E_INVAL, None, None, None, None
        if k > len(cand):
            return E_NOSPACE, None, None, None, None
        reqs = handle_requests(self.tables, self.nb, self.bph)
        handles, evicted, total = selective_handles(k, reqs, cost, cand)
        chosen = set(handles)
        inv = [(r, c, int(e)) for r, row in enumerate(self.tables) for c, e in enumerate(row)
               if e >= 0 and int(e) // self.bph in chosen]
        kept = {int(e) for r, row in enumerate(self.tables) if r not in evicted for e in row if e >= 0}
        for r in sorted(evicted):
            for e in self.tables[r]:
                if e >= 0 and int(e) not in kept:
                    self.live[int(e)] = 0
            self.tables[r, :] = -1
        for h in handles:
            self.live[h * self.bph:(h + 1) * self.bph] = 0
            self.released.append((h * self.bph, (h + 1) * self.bph))
        return OK, handles, sorted(evicted), inv, total

    def reclaim_or_evict(self, lo: int, hi: int, cost):
        """Hand (hi - lo) / bph handles to the online tenant: by emptying [lo, hi) through relocation when
        the free blocks elsewhere suffice, otherwise by evicting that many handles chosen by Algorithm 1.
        Returns (status, mode, payload): mode 0 = relocated, payload (src, dst, remap); mode 1 = evicted,
        payload (handles, evicted rows, invalidated entries, total cost)."""
        st, src, dst, remap = self.reclaim(lo, hi)
        if st == OK:
            return OK, 0, (src, dst, remap)
        if st != E_NOSPACE:
            return st, None, None
        st, handles, evicted, inv, total = self.evict((hi - lo) // self.bph, cost)
        if st != OK:
            return st, None, None
        return OK, 1, (handles, evicted, inv, total)
