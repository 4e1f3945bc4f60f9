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
        """The online tenant gives a previously released range back; its blocks become free."""
        if (lo, hi) not in self.released:
            return E_INVAL
        self.released.remove((lo, hi))
        return OK
