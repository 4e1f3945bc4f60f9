#!/usr/bin/env python3
"""Writes tests/golden/oracle_tiny_seed0.json from the CPU oracle alone.

Run from the repository root:  python tests/golden/make_oracle_golden.py
It imports only `oracle/` and the input generator `synth/`; nothing from the GPU library.
The stored numbers make a later change of the oracle's arithmetic visible (the test that reads
them fails), so that such a change has to be made on purpose and justified.
"""
import hashlib
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import synth                                                    # noqa: E402
from oracle.attention import PoolLayout, paged_decode_attention  # noqa: E402
from oracle.plan import attention_plan, prefill_plan            # noqa: E402
from oracle.prefill import paged_prefill_attention              # noqa: E402
from oracle.reclaim import ReclaimOracle                        # noqa: E402


def digest(a) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def main():
    wl = synth.workload("tiny")
    g = wl.geom
    st = synth.build_state(wl, seed=0)
    lay = PoolLayout(g.num_layers, g.num_kv_heads, g.head_dim, g.block_tokens)
    q = synth.query_bits(wl, 0, 0)
    out = paged_decode_attention(st.pool_bits, lay, q, st.tables, st.ctx_len, 0)
    picks = [(s, h, d) for s in range(wl.num_seqs) for h in (0, g.num_q_heads - 1) for d in (0, g.head_dim // 2, g.head_dim - 1)]
    q_len = np.minimum(st.ctx_len, 5).astype(np.int32)
    q_start = np.concatenate([[0], np.cumsum(q_len)[:-1]]).astype(np.int64)
    total_q = int(q_len.sum())
    pq = synth.hash_bf16_bits(np.arange(total_q * g.num_q_heads * g.head_dim, dtype=np.int64), 0, 7).reshape(
        total_q, g.num_q_heads, g.head_dim)
    pout = paged_prefill_attention(st.pool_bits, lay, pq, q_start, q_len, st.tables, st.ctx_len, 0)
    work, starts = attention_plan(st.ctx_len, g.num_kv_heads, g.head_dim, g.block_tokens, 64, 100000)
    pwork, pstarts, ptiles, pbase = prefill_plan(st.ctx_len, q_len, g.num_q_heads, g.num_kv_heads, g.head_dim,
                                                 g.block_tokens, 64, 100000)
    lo, hi = wl.reclaim_range
    orc = ReclaimOracle(g.num_blocks, g.blocks_per_handle, st.live, st.tables, None)
    status, src, dst, remap = orc.reclaim(lo, hi)
    doc = {
        "written_by": "tests/golden/make_oracle_golden.py (oracle only)",
        "workload": "tiny, seed 0, layer 0",
        "ctx_len": [int(x) for x in st.ctx_len],
        "decode_samples": [{"seq": s, "head": h, "d": d, "value": repr(float(out[s, h, d]))} for s, h, d in picks],
        "prefill_rows": total_q,
        "prefill_samples": [{"row": r, "head": h, "d": d, "value": repr(float(pout[r, h, d]))}
                            for r in (0, total_q // 2, total_q - 1) for h in (0, g.num_q_heads - 1) for d in (0, g.head_dim - 1)],
        "attention_plan": {"chunk_tokens": 64, "slice_bytes": 100000, "n_items": int(len(work)),
                           "n_slices": int(len(starts) - 1), "work_sha256": digest(np.asarray(work, dtype=np.int32))},
        "prefill_plan": {"chunk_tokens": 64, "slice_bytes": 100000, "n_items": int(len(pwork)), "n_tiles": int(len(ptiles)),
                         "work_sha256": digest(np.asarray(pwork, dtype=np.int32))},
        "reclaim": {"range": [int(lo), int(hi)], "status": int(status), "moves": [[int(a), int(b)] for a, b in zip(src, dst)],
                    "tables_sha256": digest(orc.tables.astype(np.int32)), "live_sha256": digest(orc.live.astype(np.uint8))},
    }
    path = os.path.join(ROOT, "tests", "golden", "oracle_tiny_seed0.json")
    with open(path, "w") as f:
        json.dump(doc, f, indent=1)
        f.write("\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
