"""Writes the synthetic state of a workload (geometry, context lengths, block tables, live bitmap) to
a flat little-endian file, so that a process without Python can run on exactly the contexts the
benchmark uses.  Usage: python -m synth.dump_state <workload> <seed> <out file>

Layout: 16 int32 (magic 0x53564B56, version 1, layers, query heads, kv heads, head dim, blocks,
blocks per handle, sequences, table rows, table columns, reclaim range first, reclaim range end,
chunk tokens, 0, 0), 2 int64 (slice bytes, reclamation chunk bytes), int32 context lengths
[sequences], int32 block tables [rows][columns], uint8 live flags [blocks]."""
import sys

import numpy as np

from .workload import build_state, workload

MAGIC = 0x53564B56


def dump(name: str, seed: int, path: str) -> None:
    wl = workload(name)
    g = wl.geom
    st = build_state(wl, seed, materialize_pool=False)
    lo, hi = wl.reclaim_range
    head = np.array([MAGIC, 1, g.num_layers, g.num_q_heads, g.num_kv_heads, g.head_dim, g.num_blocks,
                     g.blocks_per_handle, wl.num_seqs, st.tables.shape[0], st.tables.shape[1], lo, hi,
                     wl.chunk_tokens, 0, 0], dtype="<i4")
    with open(path, "wb") as f:
        f.write(head.tobytes())
        f.write(np.array([wl.slice_bytes, wl.chunk_bytes], dtype="<i8").tobytes())
        f.write(np.ascontiguousarray(st.ctx_len, dtype="<i4").tobytes())
        f.write(np.ascontiguousarray(st.tables, dtype="<i4").tobytes())
        f.write(np.ascontiguousarray(st.live, dtype=np.uint8).tobytes())


if __name__ == "__main__":
    if len(sys.argv) != 4:
        sys.exit(__doc__)
    dump(sys.argv[1], int(sys.argv[2]), sys.argv[3])
