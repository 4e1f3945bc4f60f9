"""Seeded workloads: pool geometry, fragmented occupancy, block tables, bf16 data.

Everything here is input construction.  The recipes stand in for the private
production workload pairs of the paper's evaluation (Section 7), which are not
available: context-length mixes, batch sizes and head shapes of LLM decode,
and a KV pool of equal-size handles (Section 3, Section 5) whose blocks are
scattered at random because KV is not contiguous inside handles (Section 5,
"Selective handle reclamation").

Data layout of the pool (one flat array of bf16 bit patterns, uint16):

    pool[block][layer][K|V][kv_head][slot][d]

so that a range of block ids is a range of addresses.

Values come from a counter-based hash of the element index, written twice with
the same integer steps (numpy for the host, torch ops for a device fill), so a
200 GiB pool can be filled on the device and any block regenerated on the host
without ever materialising the pool in host memory.
"""
from __future__ import annotations

import math
import struct
from dataclasses import dataclass, field, replace
from typing import Dict, Optional, Sequence, Tuple

import numpy as np

BF16_NAN_BITS = 0x7FC0

_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_MUL1 = 0xBF58476D1CE4E5B9
_MUL2 = 0x94D049BB133111EB
_STREAM_MUL = 0xD1B54A32D192ED03
_KEY_ADD = 0x632BE59BD9B4E019

# Sum of eight 16-bit uniforms: mean 8*65535/2, variance 8*(65536^2-1)/12.
_IH_MEAN = 4 * 65535
_IH_SCALE = struct.unpack("<f", struct.pack("<f", 1.0 / math.sqrt(8.0 * (65536.0**2 - 1.0) / 12.0)))[0]

STREAM_POOL = 0
STREAM_QUERY = 1


# --------------------------------------------------------------------------
# geometry
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Geometry:
    num_layers: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    num_blocks: int
    blocks_per_handle: int
    block_tokens: int = 16

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    @property
    def block_elems(self) -> int:
        return self.num_layers * 2 * self.num_kv_heads * self.block_tokens * self.head_dim

    @property
    def block_bytes(self) -> int:
        return 2 * self.block_elems

    @property
    def pool_elems(self) -> int:
        return self.num_blocks * self.block_elems

    @property
    def pool_bytes(self) -> int:
        return self.num_blocks * self.block_bytes

    @property
    def kv_bytes_per_token_layer(self) -> int:
        return 2 * self.num_kv_heads * self.head_dim * 2

    def elem_offset(self, block: int, layer: int, kv: int, head: int, slot: int) -> int:
        """Element index of d=0 for (block, layer, K=0|V=1, kv head, slot)."""
        o = block
        o = o * self.num_layers + layer
        o = o * 2 + kv
        o = o * self.num_kv_heads + head
        o = o * self.block_tokens + slot
        return o * self.head_dim


@dataclass(frozen=True)
class Workload:
    name: str
    geom: Geometry
    num_seqs: int
    ctx_dist: Tuple  # ("uniform", lo, hi) | ("lognormal", median, sigma, lo, cap)
    occupancy: Optional[float]  # fraction of pool blocks live; None = decode batch only
    reclaim_blocks: int  # size of the highest-address range handed to the online tenant
    chunk_bytes: int = 0  # live bytes per copy launch; 0 = one launch
    rate_cap: float = 0.0  # bytes/s of live data copied; 0 = uncapped
    slice_bytes: int = 512 << 20  # K+V bytes per attention launch; bounds the yield latency
    chunk_tokens: int = 1024  # tokens of one kv head handled by one workgroup
    shared_prefix_blocks: int = 0  # sequence 1 shares this many leading blocks with sequence 0

    @property
    def ctx_cap(self) -> int:
        return int(self.ctx_dist[2] if self.ctx_dist[0] == "uniform" else self.ctx_dist[4])

    @property
    def max_blk(self) -> int:
        return -(-self.ctx_cap // self.geom.block_tokens)

    @property
    def reclaim_range(self) -> Tuple[int, int]:
        nb = self.geom.num_blocks
        return nb - self.reclaim_blocks, nb


def _g(L, hq, hkv, d, nb, bph):
    return Geometry(num_layers=L, num_q_heads=hq, num_kv_heads=hkv, head_dim=d,
                    num_blocks=nb, blocks_per_handle=bph)


WORKLOADS: Dict[str, Workload] = {
    # The five configurations, sizes binary (GiB/MiB), rates decimal.
    "tiny": Workload("tiny", _g(1, 8, 8, 64, 256, 8), 4, ("uniform", 16, 256), 0.5, 64,
                     chunk_bytes=256 << 10, slice_bytes=256 << 10, chunk_tokens=64),
    "llama8b": Workload("llama8b", _g(32, 32, 8, 128, 20480, 32), 64,
                        ("lognormal", 2048, 0.7, 16, 8192), 0.70, 2048, slice_bytes=1 << 30),
    "offline_batch": Workload("offline_batch", _g(8, 32, 8, 128, 327680, 128), 256,
                              ("uniform", 512, 32768), None, 16384, chunk_bytes=64 << 20, rate_cap=20e9,
                              slice_bytes=1 << 30, chunk_tokens=2048),
    "llama70b_tp8": Workload("llama70b_tp8", _g(80, 8, 1, 128, 104832, 64), 128,
                             ("lognormal", 4096, 0.7, 16, 16384), 0.85, 13120, slice_bytes=1 << 30,
                             chunk_tokens=1408),
    "stress": Workload("stress", _g(10, 32, 8, 128, 327680, 64), 512,
                       ("uniform", 256, 16384), 0.90, 26240, slice_bytes=1 << 30, chunk_tokens=2048),
    # Reduced shapes (same heads, fewer layers / sequences / blocks) that a CPU
    # oracle finishes in seconds yet span several chunks, slices and ragged tails.
    "llama8b_small": Workload("llama8b_small", _g(2, 32, 8, 128, 2048, 32), 8,
                              ("lognormal", 1024, 0.7, 16, 4096), 0.70, 512,
                              chunk_bytes=8 << 20, slice_bytes=4 << 20),
    "offline_batch_small": Workload("offline_batch_small", _g(2, 32, 8, 128, 2560, 64), 6,
                                    ("uniform", 512, 4096), None, 256,
                                    chunk_bytes=4 << 20, rate_cap=2e9, slice_bytes=4 << 20),
    "llama70b_tp8_small": Workload("llama70b_tp8_small", _g(3, 8, 1, 128, 4096, 64), 12,
                                   ("lognormal", 2048, 0.7, 16, 8192), 0.85, 512,
                                   chunk_bytes=2 << 20, slice_bytes=2 << 20),
    "stress_small": Workload("stress_small", _g(2, 32, 8, 128, 1536, 64), 10,
                             ("uniform", 256, 2048), 0.90, 128,
                             chunk_bytes=4 << 20, slice_bytes=2 << 20),
}


def workload(name: str, **overrides) -> Workload:
    w = WORKLOADS[name]
    return replace(w, **overrides) if overrides else w


# --------------------------------------------------------------------------
# counter-based bf16 values
# --------------------------------------------------------------------------
def _key(seed: int, stream: int) -> int:
    return (seed * _GOLDEN + stream * _STREAM_MUL + _KEY_ADD) & _M64


def _mix64_np(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * np.uint64(_MUL1)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(_MUL2)
    return z ^ (z >> np.uint64(31))


def _fields_sum_np(z: np.ndarray) -> np.ndarray:
    m = np.uint64(0xFFFF)
    return ((z & m) + ((z >> np.uint64(16)) & m) + ((z >> np.uint64(32)) & m)
            + (z >> np.uint64(48))).astype(np.int64)


def hash_bf16_bits(idx: np.ndarray, seed: int, stream: int = STREAM_POOL) -> np.ndarray:
    """bf16 bit patterns (uint16), approximately N(0,1), for element indices `idx`."""
    with np.errstate(over="ignore"):
        z0 = np.asarray(idx).astype(np.uint64) ^ np.uint64(_key(seed, stream))
        z1 = _mix64_np(z0)
        z2 = _mix64_np(z1 + np.uint64(_GOLDEN))
    s = _fields_sum_np(z1) + _fields_sum_np(z2) - _IH_MEAN
    x = s.astype(np.float32) * np.float32(_IH_SCALE)
    u = x.view(np.uint32)
    u = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return u.astype(np.uint16)


def _s64(c: int) -> int:
    c &= _M64
    return c - (1 << 64) if c >= (1 << 63) else c


def _lsr_t(z, k: int):
    return (z >> k) & ((1 << (64 - k)) - 1)


def _mix64_t(z):
    z = (z ^ _lsr_t(z, 30)) * _s64(_MUL1)
    z = (z ^ _lsr_t(z, 27)) * _s64(_MUL2)
    return z ^ _lsr_t(z, 31)


def _fields_sum_t(z):
    return (z & 0xFFFF) + ((z >> 16) & 0xFFFF) + ((z >> 32) & 0xFFFF) + ((z >> 48) & 0xFFFF)


def hash_bf16_bits_torch(idx, seed: int, stream: int = STREAM_POOL):
    """Same values as `hash_bf16_bits`, from an int64 torch tensor (any device); int16 out."""
    import torch

    z0 = idx ^ _s64(_key(seed, stream))
    z1 = _mix64_t(z0)
    z2 = _mix64_t(z1 + _s64(_GOLDEN))
    s = _fields_sum_t(z1) + _fields_sum_t(z2) - _IH_MEAN
    x = s.to(torch.float32) * _IH_SCALE
    u = x.view(torch.int32)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16  # finite inputs: arithmetic shift then mask below
    u = ((u & 0xFFFF) ^ 0x8000) - 0x8000  # fold into the int16 range before narrowing
    return u.to(torch.int16)


def pool_bits_for_blocks(geom: Geometry, seed: int, block_ids: Sequence[int]) -> np.ndarray:
    """uint16 [len(block_ids), block_elems]: the hash contents of the given blocks."""
    be = geom.block_elems
    ids = np.asarray(block_ids, dtype=np.int64)
    out = np.empty((len(ids), be), dtype=np.uint16)
    lane = np.arange(be, dtype=np.int64)
    for i, b in enumerate(ids):
        out[i] = hash_bf16_bits(lane + int(b) * be, seed, STREAM_POOL)
    return out


def fill_pool_range_torch(pool_i16, geom: Geometry, seed: int, first: int, last: int,
                          chunk_elems: int = 1 << 26) -> None:
    """Fill elements [first, last) of a flat int16 torch tensor of pool_elems elements in place."""
    import torch

    assert pool_i16.numel() >= geom.pool_elems and pool_i16.dtype == torch.int16
    assert 0 <= first <= last <= geom.pool_elems
    flat = pool_i16.view(-1)
    for lo in range(first, last, chunk_elems):
        hi = min(last, lo + chunk_elems)
        idx = torch.arange(lo, hi, dtype=torch.int64, device=flat.device)
        flat[lo:hi] = hash_bf16_bits_torch(idx, seed, STREAM_POOL)


def fill_pool_torch(pool_i16, geom: Geometry, seed: int, chunk_elems: int = 1 << 26) -> None:
    """Fill a flat int16 torch tensor of pool_elems elements in place (device or host)."""
    fill_pool_range_torch(pool_i16, geom, seed, 0, geom.pool_elems, chunk_elems)


def query_bits(wl: Workload, seed: int, layer: int) -> np.ndarray:
    """uint16 [S, Hq, D] bf16 bit patterns of the decode queries of one layer."""
    g = wl.geom
    n = wl.num_seqs * g.num_q_heads * g.head_dim
    idx = np.arange(n, dtype=np.int64) + layer * n
    return hash_bf16_bits(idx, seed, STREAM_QUERY).reshape(wl.num_seqs, g.num_q_heads, g.head_dim)


# --------------------------------------------------------------------------
# pool occupancy, block tables
# --------------------------------------------------------------------------
@dataclass
class PoolState:
    wl: Workload
    seed: int
    ctx_len: np.ndarray            # int32 [S]
    tables: np.ndarray             # int32 [n_rows, max_blk]; rows < S are the decode batch
    live: np.ndarray               # uint8 [NB]
    pool_bits: Optional[np.ndarray] = None  # uint16 [NB*block_elems] when materialised
    poisoned: list = field(default_factory=list)  # (block, first_unused_slot) pairs

    @property
    def geom(self) -> Geometry:
        return self.wl.geom

    @property
    def n_rows(self) -> int:
        return self.tables.shape[0]

    @property
    def max_blk(self) -> int:
        return self.tables.shape[1]


def sample_ctx_len(wl: Workload, rng: np.random.Generator) -> np.ndarray:
    kind = wl.ctx_dist[0]
    if kind == "uniform":
        _, lo, hi = wl.ctx_dist
        n = rng.integers(lo, hi + 1, size=wl.num_seqs)
    elif kind == "lognormal":
        _, median, sigma, lo, cap = wl.ctx_dist
        n = np.rint(rng.lognormal(math.log(median), sigma, size=wl.num_seqs))
        n = np.clip(n, lo, cap)
    else:
        raise ValueError(kind)
    return n.astype(np.int32)


def build_state(wl: Workload, seed: int, materialize_pool: bool = True,
                poison_unused: bool = True) -> PoolState:
    """Context lengths, a random live subset of the pool, and block tables.

    live = uniformly random subset of round(occupancy*NB) block ids; the decode
    batch takes its blocks from that subset in permuted order (so logically
    consecutive blocks are physically scattered); the rest are "background"
    blocks of sequences outside the batch, listed in table rows after the batch.
    """
    g = wl.geom
    rng = np.random.Generator(np.random.PCG64(seed))
    ctx = sample_ctx_len(wl, rng)
    nblk = -(-ctx.astype(np.int64) // g.block_tokens)
    shared = wl.shared_prefix_blocks
    if shared:
        assert wl.num_seqs >= 2 and nblk[0] >= shared and nblk[1] >= shared
    own = nblk.copy()
    if shared:
        own[1] -= shared
    batch_blocks = int(own.sum())
    n_live = batch_blocks if wl.occupancy is None else max(batch_blocks, int(round(wl.occupancy * g.num_blocks)))
    if n_live > g.num_blocks:
        raise ValueError(f"{wl.name}: batch needs {n_live} blocks, pool has {g.num_blocks}")
    perm = rng.permutation(g.num_blocks).astype(np.int32)
    live_ids = perm[:n_live]
    live = np.zeros(g.num_blocks, dtype=np.uint8)
    live[live_ids] = 1

    max_blk = wl.max_blk
    n_bg = n_live - batch_blocks
    bg_rows = -(-n_bg // max_blk)
    tables = np.full((wl.num_seqs + bg_rows, max_blk), -1, dtype=np.int32)
    cur = 0
    for s in range(wl.num_seqs):
        if shared and s == 1:
            tables[1, :shared] = tables[0, :shared]
            tables[1, shared:nblk[1]] = live_ids[cur:cur + own[1]]
        else:
            tables[s, :nblk[s]] = live_ids[cur:cur + own[s]]
        cur += int(own[s])
    for r in range(bg_rows):
        take = min(max_blk, n_live - cur)
        tables[wl.num_seqs + r, :take] = live_ids[cur:cur + take]
        cur += take
    assert cur == n_live

    st = PoolState(wl=wl, seed=seed, ctx_len=ctx, tables=tables, live=live)
    for s in range(wl.num_seqs):
        used = int(ctx[s]) % g.block_tokens
        if used:
            st.poisoned.append((int(tables[s, nblk[s] - 1]), used))
    if materialize_pool:
        idx = np.arange(g.pool_elems, dtype=np.int64)
        st.pool_bits = hash_bf16_bits(idx, seed, STREAM_POOL)
        if poison_unused:
            poison_unused_slots(st, st.pool_bits)
    return st


def unused_slot_spans(st: PoolState):
    """(start_elem, n_elems) runs covering never-read slots of each batch sequence's last block."""
    g = st.geom
    for blk, used in st.poisoned:
        for layer in range(g.num_layers):
            for kv in (0, 1):
                for h in range(g.num_kv_heads):
                    o = g.elem_offset(blk, layer, kv, h, used)
                    yield o, (g.block_tokens - used) * g.head_dim


def poison_unused_slots(st: PoolState, pool_flat) -> None:
    """Write bf16 NaN into slots past each sequence's length (numpy uint16 or torch int16, flat)."""
    g = st.geom
    shape = (g.num_blocks, g.num_layers, 2, g.num_kv_heads, g.block_tokens, g.head_dim)
    n = g.pool_elems
    view = pool_flat[:n].reshape(shape) if isinstance(pool_flat, np.ndarray) else pool_flat[:n].view(shape)
    for blk, used in st.poisoned:
        view[blk, :, :, :, used:, :] = BF16_NAN_BITS
