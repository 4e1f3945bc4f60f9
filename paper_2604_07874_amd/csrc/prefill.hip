// Preemptible causal attention of a chunk of new tokens over the paged KV pool (prefill).
//
// Long prefills are where coarse preemption costs most (paper Section 2.2: layer-level
// preemption delays of hundreds of milliseconds at 32k tokens; Section 5: bursts arriving
// during a long prefill iteration).  The same slicing as for decode bounds the time to the
// next yield point; here the work is compute-bound, so the MFMA units carry the load.
//
// Work split: the new tokens of a sequence are cut into query tiles of 128/GP positions
// (GP = group size rounded up to a power of two), so a tile has 128 (position, query head)
// columns; the tokens a tile can see (positions 0 .. its last position) are cut into chunks
// of chunk_tokens; one work item = (tile, kv head, chunk) = one workgroup.  Items of a tile
// are merged by a separate small kernel after the layer's last slice (prefill launches last
// milliseconds, so one more launch per layer is immaterial and needs no in-kernel
// cross-workgroup ordering).
//
// Kernel shape (wave64, gfx950): 4 waves; wave w owns columns [32w, 32w+32) as two 16-column
// MFMA tiles and sees every token of the item.  Per 32-token group the workgroup brings K and V
// into LDS once for all four waves, with the 16-byte global->LDS loads of gfx950: wave w asks
// for rows 4w .. 4w+3 of both blocks of the group, K and V, four loads in all, which need no
// registers and are requested three groups ahead of their use.  The rows lie in LDS as in the
// pool (256 bytes per token), their 16-byte chunks permuted so that the operand reads meet no
// bank conflict.  After the step's barrier each wave reads the 8 K operands (16-byte reads) and
// the 8 V operands (transposing 8-byte reads, which hand each lane its own head dimension of
// four tokens) it needs for its MFMAs (v_mfma_f32_16x16x32_bf16) and runs online softmax per
// column with the causal mask applied by select.
#include "vkv_internal.h"

#include <algorithm>
#include <cmath>
#include <cstring>

namespace vkv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kTileColumns = 128;   // (position, query head) columns of one query tile
constexpr int kNQ = 2;              // 16-column MFMA tiles per wave
constexpr int kMaxPrefillChunkTokens = 16384;   // bounds an item's run time, not a kernel limit
constexpr float kSlack = 8.0f;      // how far (log2 units) a score may exceed the running reference
constexpr float kNoMax = -1.0e30f;  // reference of a column that has seen no token yet (finite on purpose)

struct PrefillParams {
  const uint16_t* pool;       // pool base + layer offset (elements)
  const WorkItem* work;       // .seq = tile id
  const int32_t* tiles;       // [n_tiles][4] = (sequence, first q row, first position, positions)
  const int32_t* tile_base;   // [n_tiles + 1]
  const int32_t* order;       // [n_items] launch order: within a slice, items by falling token count
  const int32_t* merge_tiles; // tiles that were split into several chunks
  const uint16_t* q;          // [total_q][Hq][D]
  const int32_t* table;
  float* part_acc;            // [n_items][128][D]
  float* part_ml;             // [n_items][128][2]
  float* out;                 // [total_q][Hq][D]
  uint32_t* err;
  uint64_t block_elems;
  uint32_t v_off;
  int32_t item_first, max_blk, Hq, Hkv, G, gp_shift, NB;
  float scale_log2;
};

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// LDS reads the compiler does not see as such.  It orders every LDS read it knows of behind all pending
// global->LDS loads (it cannot tell the staging buffers apart), which would wait for the groups that were
// requested ahead; these reads are ordered by hand instead: the loads of a buffer are waited for
// (s_waitcnt vmcnt) before the barrier that lets anyone read it.
template <int OFF>
__device__ __forceinline__ void lds_read_b128(u32x4& dst, uint32_t addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
// transposing 8-byte read: within 16 lanes, lane i gets element i & 3 of the four 16-bit elements that lane
// 4 j + (i >> 2) points at, for j = 0..3
template <int OFF>
__device__ __forceinline__ void lds_read_tr16_b64(u32x2& dst, uint32_t addr) {
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
__device__ __forceinline__ void lds_wait(u32x4 (&a)[8]) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7])
               :: "memory");
}
__device__ __forceinline__ void lds_wait(u32x2 (&a)[16]) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7]),
                 "+v"(a[8]), "+v"(a[9]), "+v"(a[10]), "+v"(a[11]), "+v"(a[12]), "+v"(a[13]), "+v"(a[14]), "+v"(a[15])
               :: "memory");
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

template <int D>
__global__ __launch_bounds__(256, 2) void paged_prefill_attn_slice_kernel(const PrefillParams p) {
  static_assert(D == 128, "head_dim 128 only");
  constexpr int EPL = D / 16;
  constexpr int KS = D / 32;
  constexpr int ROW = D * 2;            // bytes of one token row of one head
  constexpr float NEG_INF = -INFINITY;

  // Four staging buffers of a 32-token group each, K rows and V rows as they lie in the pool (256 bytes
  // per token), written by the 16-byte global->LDS loads; no padding is possible there (a load places its
  // 64 lanes back to back), so the 16-byte chunks of a row are permuted instead, by the choice of the
  // global address each lane asks for: chunk c of K row r sits at position c ^ (r & 15), chunk c of V row r
  // at c ^ 2 (r & 7) (the LDS has 64 banks: 16 lanes of a 16-byte read, 32 lanes of an 8-byte read go together).
  constexpr int kBufs = 4;
  __shared__ __attribute__((aligned(16))) unsigned char k_lds4[kBufs][32 * ROW];
  __shared__ __attribute__((aligned(16))) unsigned char v_lds4[kBufs][32 * ROW];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c16 = lane & 15, kg = lane >> 4;

  const int item_id = p.order[p.item_first + blockIdx.x];   // longest items of the slice start first
  const WorkItem it = p.work[item_id];
  const int tile = it.seq;
  const int seq = p.tiles[4 * tile + 0], row0 = p.tiles[4 * tile + 1], pos0 = p.tiles[4 * tile + 2],
            n_pos = p.tiles[4 * tile + 3];
  const int ntok = it.n_tokens;
  const int tok_base = it.first_block * 16;          // position of the item's first token
  const int ngroups = (ntok + kGroupTokens - 1) / kGroupTokens;
  const int G = p.G, gp_mask = (1 << p.gp_shift) - 1;

  // this lane's two columns (one per MFMA tile): position within the tile and query head
  int cpos[kNQ], cg[kNQ];
  bool cvalid[kNQ];
  bf16x8 qb[kNQ][KS];
#pragma unroll
  for (int j = 0; j < kNQ; ++j) {
    const int col = (wave * kNQ + j) * 16 + c16;
    cpos[j] = col >> p.gp_shift;
    cg[j] = col & gp_mask;
    cvalid[j] = cg[j] < G && cpos[j] < n_pos;
    const uint16_t* qrow = p.q + ((size_t)(row0 + (cvalid[j] ? cpos[j] : 0)) * p.Hq + (size_t)it.kv_head * G +
                                  (cvalid[j] ? cg[j] : 0)) * D;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (cvalid[j]) v = *reinterpret_cast<const u32x4*>(qrow + ks * 32 + kg * 8);
      qb[j][ks] = __builtin_bit_cast(bf16x8, v);
    }
  }

  const int32_t* trow = p.table + (size_t)seq * p.max_blk + it.first_block;
  const unsigned char* kplane = reinterpret_cast<const unsigned char*>(p.pool + (size_t)it.kv_head * (16 * D));
  const int nblk_item = (ntok + 15) >> 4;
  // Byte offsets of the item's blocks from kplane, 64 at a time, one per lane: lane i of (o0lo, o0hi) holds
  // entry 64 win + i, (o1lo, o1hi) the 64 after those.  An entry past the item's end or outside the pool
  // (a corrupted table, reported here) gets hi = -1; the loads then go to the item's latest good block,
  // whose rows exist, and what they bring is masked (K) or cleared after it is read (V).
  uint32_t o0lo, o0hi, o1lo, o1hi;
  auto window = [&](int w, uint32_t& lo, uint32_t& hi) {
    const int e = w * 64 + lane;
    int32_t blk = -1;
    if (e < nblk_item) {
      blk = trow[e];
      if (blk < 0 || blk >= p.NB) {
        atomicOr(p.err, 1u);
        blk = -1;
      }
    }
    const uint64_t off = (uint64_t)(uint32_t)blk * (p.block_elems * 2);
    lo = (uint32_t)off;
    hi = blk < 0 ? 0xFFFFFFFFu : (uint32_t)(off >> 32);
    // have it now: no load with a register result is then pending from one step to the next, and the
    // compiler has no reason to wait for the loads into LDS along with it
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(lo), "+v"(hi) :: "memory");
  };
  window(0, o0lo, o0hi);
  window(1, o1lo, o1hi);
  int win = 0;
  // the item's first block must be good: there is nothing to fall back on before it
  uint32_t safe_lo = __builtin_amdgcn_readlane(o0lo, 0), safe_hi = __builtin_amdgcn_readlane(o0hi, 0);
  if (safe_hi == 0xFFFFFFFFu) return;   // reported above; the whole workgroup leaves, before any barrier

  f32x4 acc[kNQ][EPL], accl[kNQ];
  float m_run[kNQ];
#pragma unroll
  for (int j = 0; j < kNQ; ++j) {
    m_run[j] = kNoMax;
    accl[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int dt = 0; dt < EPL; ++dt) acc[j][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  bf16x8 ones;
#pragma unroll
  for (int i = 0; i < 8; ++i) ones[i] = (__bf16)1.0f;
  // last token index (within the item) that every column of this wave may see
  const int wave_limit = pos0 + ((wave * kNQ * 16) >> p.gp_shift) - tok_base;

  // ---- this wave's share of a group goes from the pool straight into LDS ----
  // Rows 4 wave .. 4 wave + 3 of both blocks of the group, K and V: four loads of 64 x 16 bytes.  Lane l
  // fills position l & 15 of row 4 wave + (l >> 4), so it asks for the chunk that belongs there.
  const int lrow = 4 * wave + kg;                                     // row within a block
  const uint32_t g_off_k = (uint32_t)(lrow * ROW + ((c16 ^ (lrow & 15)) * 16));        // bytes
  const uint32_t g_off_v = (uint32_t)(lrow * ROW + ((c16 ^ (2 * (lrow & 7))) * 16));
  const uint64_t v_bytes = (uint64_t)p.v_off * 2;
  auto issue = [&](int grp) {
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
      const int bi = grp * 2 + sb;
      if ((bi >> 6) != win) {   // blocks are visited in rising order, so the window moves one step at a time
        win = bi >> 6;
        o0lo = o1lo;
        o0hi = o1hi;
        window(win + 1, o1lo, o1hi);
      }
      uint32_t lo = __builtin_amdgcn_readlane(o0lo, bi & 63), hi = __builtin_amdgcn_readlane(o0hi, bi & 63);
      const bool good = hi != 0xFFFFFFFFu;
      lo = good ? lo : safe_lo;
      hi = good ? hi : safe_hi;
      safe_lo = lo;
      safe_hi = hi;
      const unsigned char* src = kplane + (((uint64_t)hi << 32) | lo);
      unsigned char* kd = k_lds4[grp & (kBufs - 1)] + (sb * 16 + 4 * wave) * ROW;
      unsigned char* vd = v_lds4[grp & (kBufs - 1)] + (sb * 16 + 4 * wave) * ROW;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + g_off_k),
                                       (__attribute__((address_space(3))) void*)kd, 16, 0, 0);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + v_bytes + g_off_v),
                                       (__attribute__((address_space(3))) void*)vd, 16, 0, 0);
    }
  };
  // all of this wave's loads but those of the newest group (four, if there is one) have landed
  auto wait_all_but = [&](bool one_group) {
    if (one_group) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  };

  // ---- q.K of a staged group for both column tiles of this wave ----
  // row c16 of the K operand is token 16 b + c16 of the group; its chunk ks 4 + kg sits at (ks 4 + kg) ^ c16
  uint32_t k_addr[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) k_addr[ks] = lds_addr(&k_lds4[0][0]) + c16 * ROW + (((ks * 4 + kg) ^ c16) << 4);
  auto scores = [&](int grp, f32x4 (&sc)[kNQ][2]) {
    const uint32_t boff = (uint32_t)(grp & (kBufs - 1)) * (32 * ROW);
    u32x4 ka[8];   // [b * KS + ks]
    lds_read_b128<0>(ka[0], k_addr[0] + boff);
    lds_read_b128<16 * ROW>(ka[4], k_addr[0] + boff);
    lds_read_b128<0>(ka[1], k_addr[1] + boff);
    lds_read_b128<16 * ROW>(ka[5], k_addr[1] + boff);
    lds_read_b128<0>(ka[2], k_addr[2] + boff);
    lds_read_b128<16 * ROW>(ka[6], k_addr[2] + boff);
    lds_read_b128<0>(ka[3], k_addr[3] + boff);
    lds_read_b128<16 * ROW>(ka[7], k_addr[3] + boff);
    lds_wait(ka);
#pragma unroll
    for (int j = 0; j < kNQ; ++j)
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        sc[j][b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          sc[j][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[b * KS + ks]), qb[j][ks],
                                                             sc[j][b], 0, 0, 0);
      }
  };
  // ---- softmax of a group's scores and its p.V products ----
  // The V operand of d-tile dt (d = 16 dt + c16 in this lane) comes from two transposing reads, one per
  // block of the group: the 16 lanes of a k-group point at 8-byte pieces of rows 4 kg .. 4 kg + 3 (lane s
  // at row 4 kg + (s >> 2), d = 16 dt + 4 (s & 3)) and each gets its own d of those four rows back.
  const int v_rr = c16 >> 2, v_q = c16 & 3;
  const int v_base = (4 * kg + v_rr) * ROW + v_q * 8;
  const int v_sw = (4 * kg + v_rr) & 7;
  uint32_t v_addr[EPL];
#pragma unroll
  for (int dt = 0; dt < EPL; ++dt) v_addr[dt] = lds_addr(&v_lds4[0][0]) + v_base + ((dt ^ v_sw) << 5);
  auto finish = [&](int grp, f32x4 (&sc)[kNQ][2]) {
    const int tok0 = grp * kGroupTokens;
    const uint32_t boff = (uint32_t)(grp & (kBufs - 1)) * (32 * ROW);
    // requested first, so that they arrive while the softmax below is computed
    u32x2 vh[16];   // [2 dt + block of the group]
#define VKV_VREAD(dt) lds_read_tr16_b64<0>(vh[2 * dt], v_addr[dt] + boff); lds_read_tr16_b64<16 * ROW>(vh[2 * dt + 1], v_addr[dt] + boff);
    VKV_VREAD(0) VKV_VREAD(1) VKV_VREAD(2) VKV_VREAD(3) VKV_VREAD(4) VKV_VREAD(5) VKV_VREAD(6) VKV_VREAD(7)
#undef VKV_VREAD
    // A group is interior for this wave when every token of it exists and is visible to every column of
    // the wave; only the groups on the causal diagonal and a ragged last group need the mask.
    const bool interior = tok0 + kGroupTokens <= ntok && tok0 + kGroupTokens - 1 <= wave_limit;
    bf16x8 pbs[kNQ];
#pragma unroll
    for (int j = 0; j < kNQ; ++j) {
      if (!interior) {
        // column = (position cpos[j], head cg[j]); token tok0 + 16b + 4kg + r sits at position tok_base + that
        const int limit = min(pos0 + cpos[j] - tok_base, ntok - 1);   // last visible token index within the item
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (tok0 + b * 16 + 4 * kg + r > limit) sc[j][b][r] = NEG_INF;   // also drops NaN from rows past the end
      }
      const float mx = fmaxf(fmaxf(fmaxf(sc[j][0][0], sc[j][0][1]), fmaxf(sc[j][0][2], sc[j][0][3])),
                             fmaxf(fmaxf(sc[j][1][0], sc[j][1][1]), fmaxf(sc[j][1][2], sc[j][1][3])));
      if (__builtin_amdgcn_ballot_w64(fmaf(mx, p.scale_log2, -kSlack) > m_run[j]) != 0ull) {
        float mc = fmaxf(mx, __shfl_xor(mx, 16));
        mc = fmaxf(mc, __shfl_xor(mc, 32));
        const float m_new = fmaxf(m_run[j], mc * p.scale_log2);
        const float alpha = __builtin_amdgcn_exp2f(m_run[j] - m_new);
        m_run[j] = m_new;
        accl[j] *= alpha;
#pragma unroll
        for (int dt = 0; dt < EPL; ++dt) acc[j][dt] *= alpha;
      }
#pragma unroll
      for (int i = 0; i < 8; ++i)
        pbs[j][i] = (__bf16)__builtin_amdgcn_exp2f(fmaf(sc[j][i >> 2][i & 3], p.scale_log2, -m_run[j]));
    }
    lds_wait(vh);
    u32x4 va[EPL];
#pragma unroll
    for (int dt = 0; dt < EPL; ++dt) va[dt] = u32x4{vh[2 * dt][0], vh[2 * dt][1], vh[2 * dt + 1][0], vh[2 * dt + 1][1]};
    if (tok0 + kGroupTokens > ntok) {
      // the item's ragged last group: rows past the end hold whatever the pool holds there (maybe NaN);
      // their weights are zero, their V must be too.  Element i of the operand is token 16 (i >> 2) + 4 kg + (i & 3).
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (tok0 + (i >> 2) * 16 + 4 * kg + (i & 3) >= ntok)
#pragma unroll
          for (int dt = 0; dt < EPL; ++dt) va[dt][i >> 1] &= (i & 1) ? 0x0000FFFFu : 0xFFFF0000u;
    }
#pragma unroll
    for (int j = 0; j < kNQ; ++j) {
      // the row sums come from the matrix unit too (a tile of ones as the "V" operand), so the
      // denominator sums exactly the rounded weights the numerator uses
      accl[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pbs[j], accl[j], 0, 0, 0);
#pragma unroll
      for (int dt = 0; dt < EPL; ++dt)
        acc[j][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, va[dt]), pbs[j], acc[j][dt], 0, 0, 0);
    }
  };

  // Software pipeline over the groups.  Loads run three groups ahead of the p.V products and need no
  // registers; the one barrier of a step says two things: every wave's loads of group g+1 have landed
  // (each wave waits for its own first), and every wave is done with step g-1, whose buffers the loads
  // issued right after the barrier overwrite.
  issue(0);
  if (1 < ngroups) issue(1);
  wait_all_but(1 < ngroups);     // group 0 has landed
  __syncthreads();
  f32x4 sc_cur[kNQ][2], sc_next[kNQ][2];
  scores(0, sc_cur);
  if (2 < ngroups) issue(2);
  for (int grp = 0; grp < ngroups; ++grp) {
    wait_all_but(grp + 2 < ngroups);   // everything up to group grp+1
    // the barrier alone, without the fence of __syncthreads: that fence would wait for the loads of the
    // two groups ahead as well; this wave's LDS reads of the previous step have returned (they fed its
    // matrix instructions), which is all the others need to know before they overwrite those buffers
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (grp + 3 < ngroups) issue(grp + 3);
    if (grp + 1 < ngroups) scores(grp + 1, sc_next);
    finish(grp, sc_cur);
#pragma unroll
    for (int j = 0; j < kNQ; ++j)
#pragma unroll
      for (int b = 0; b < 2; ++b) sc_cur[j][b] = sc_next[j][b];
  }

  // ---- results: column-owned, no merge across waves; register r of d-tile dt is d = 16 dt + 4 kg + r ----
  const int nch = (p.tile_base[tile + 1] - p.tile_base[tile]) / p.Hkv;
  const size_t item = (size_t)item_id;
#pragma unroll
  for (int j = 0; j < kNQ; ++j) {
    const float l = accl[j][0];   // every row of the ones-tile product holds the column's sum
    const int col = (wave * kNQ + j) * 16 + c16;
    if (nch == 1) {
      if (cvalid[j]) {
        float* orow = p.out + ((size_t)(row0 + cpos[j]) * p.Hq + (size_t)it.kv_head * G + cg[j]) * D;
        const float inv = 1.0f / l;
#pragma unroll
        for (int dt = 0; dt < EPL; ++dt)
          *reinterpret_cast<f32x4*>(orow + 16 * dt + 4 * kg) = acc[j][dt] * inv;
      }
    } else {
      float* prow = p.part_acc + (item * kTileColumns + col) * D;
#pragma unroll
      for (int dt = 0; dt < EPL; ++dt) *reinterpret_cast<f32x4*>(prow + 16 * dt + 4 * kg) = acc[j][dt];
      if (kg == 0) {
        p.part_ml[(item * kTileColumns + col) * 2 + 0] = m_run[j];
        p.part_ml[(item * kTileColumns + col) * 2 + 1] = l;
      }
    }
  }
}

// Merge of the chunks of one split (tile, kv head): log-sum-exp merge in chunk order.  A workgroup
// takes a quarter of the tile's columns (kMergeCols), so that a merge step has four times the
// workgroups and a quarter of the dependent loads per thread: the kernel is nothing but memory latency.
// Pass 1, one thread per column: the maximum over the chunks, then the chunk weights 2^(m_c - M)
// into LDS (32 chunks at a time) and their weighted sum of the partial sums.
// Pass 2, one thread per (column, four output dims): the weighted partial accumulators, with the
// loads of four chunks in flight at a time.
constexpr int kMergeCols = 32;
template <int D>
__global__ __launch_bounds__(256) void prefill_merge_kernel(const PrefillParams p) {
  constexpr int kBatch = 32;
  constexpr int kParts = kTileColumns / kMergeCols;
  __shared__ float sm_w[kBatch][kMergeCols];
  __shared__ float sm_M[kMergeCols], sm_den[kMergeCols];
  // item_first = first entry of the step in the list of split tiles
  const int unit = blockIdx.x / kParts, col0 = (blockIdx.x % kParts) * kMergeCols;
  const int tile = p.merge_tiles[p.item_first + unit / p.Hkv], head = unit % p.Hkv;
  const int base = p.tile_base[tile];
  const int nch = (p.tile_base[tile + 1] - base) / p.Hkv;
  const int row0 = p.tiles[4 * tile + 1], n_pos = p.tiles[4 * tile + 3];
  const int G = p.G, gp_mask = (1 << p.gp_shift) - 1;
  auto item_col = [&](int c, int col) { return ((size_t)base + (size_t)c * p.Hkv + head) * kTileColumns + col; };
  const int tid = threadIdx.x;
  if (tid < kMergeCols) {
    float M = -INFINITY;
    for (int c = 0; c < nch; ++c) M = fmaxf(M, p.part_ml[item_col(c, col0 + tid) * 2]);
    sm_M[tid] = M;
    sm_den[tid] = 0.f;
  }
  constexpr int VPR = D / 4;                         // float4 per column
  constexpr int kIters = kMergeCols * VPR / 256;
  f32x4 num[kIters];
#pragma unroll
  for (int i = 0; i < kIters; ++i) num[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int c0 = 0; c0 < nch; c0 += kBatch) {
    const int nb = min(kBatch, nch - c0);
    __syncthreads();                                 // sm_M ready / previous batch's weights consumed
    if (tid < kMergeCols) {
      const float M = sm_M[tid];
      float den = sm_den[tid];
      for (int j = 0; j < nb; ++j) {
        const size_t ic = item_col(c0 + j, col0 + tid);
        const float wt = __builtin_exp2f(p.part_ml[ic * 2] - M);   // 0 for a chunk this column cannot see
        sm_w[j][tid] = wt;
        den += wt * p.part_ml[ic * 2 + 1];
      }
      sm_den[tid] = den;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kIters; ++i) {
      const int e = i * 256 + tid, lc = e / VPR, v = e - lc * VPR;
      int j = 0;
      for (; j + 4 <= nb; j += 4) {
        f32x4 x[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
          x[u] = *reinterpret_cast<const f32x4*>(p.part_acc + item_col(c0 + j + u, col0 + lc) * D + v * 4);
#pragma unroll
        for (int u = 0; u < 4; ++u) num[i] += sm_w[j + u][lc] * x[u];
      }
      for (; j < nb; ++j)
        num[i] += sm_w[j][lc] * *reinterpret_cast<const f32x4*>(p.part_acc + item_col(c0 + j, col0 + lc) * D + v * 4);
    }
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kIters; ++i) {
    const int e = i * 256 + tid, lc = e / VPR, v = e - lc * VPR;
    const int col = col0 + lc;
    const int cpos = col >> p.gp_shift, cg = col & gp_mask;
    if (cg >= G || cpos >= n_pos) continue;
    const float inv = 1.0f / sm_den[lc];
    *reinterpret_cast<f32x4*>(p.out + ((size_t)(row0 + cpos) * p.Hq + (size_t)head * G + cg) * D + v * 4) = num[i] * inv;
  }
}

// ---- host ---------------------------------------------------------------------------

static int pf_check_bound(vkv_pool* p, const void* workspace, const char* who) {
  if (!p) { set_error("%s: null pool", who); return VKV_E_INVAL; }
  if (p->broken) { set_error("%s: pool unusable after a HIP failure", who); return VKV_E_HIP; }
  if (!p->pf.has_plan) { set_error("%s: no plan; call kv_prefill_plan first", who); return VKV_E_STATE; }
  if (!workspace || workspace != p->pf.bound_ws || p->pf.bound_gen != p->pf.gen) {
    set_error("%s: workspace is not bound to the current plan; call kv_prefill_bind", who);
    return VKV_E_STATE;
  }
  return VKV_OK;
}

static int pf_check_args(vkv_pool* p, int32_t layer, const void* q, const int32_t* table, int32_t max_blk,
                         void* workspace, void* out, const char* who) {
  int st = pf_check_bound(p, workspace, who);
  if (st != VKV_OK) return st;
  if (!p->cfg.base) { set_error("%s: pool has no device memory", who); return VKV_E_INVAL; }
  if (p->cfg.head_dim != 128) { set_error("%s: prefill supports head_dim 128 only", who); return VKV_E_INVAL; }
  if (layer < 0 || layer >= p->cfg.num_layers) { set_error("%s: layer %d out of range", who, layer); return VKV_E_INVAL; }
  if (!q || !table || !out || (uintptr_t)q % 16 || (uintptr_t)out % 16) {
    set_error("%s: q, out (16-byte aligned) and block_table must be given", who);
    return VKV_E_INVAL;
  }
  if (max_blk < p->pf.max_ctx_blocks) {
    set_error("%s: block table has %d columns, the plan needs %d", who, max_blk, p->pf.max_ctx_blocks);
    return VKV_E_INVAL;
  }
  return VKV_OK;
}

static PrefillParams pf_params(vkv_pool* p, int32_t layer, const void* q, const int32_t* table, int32_t max_blk,
                               void* workspace, void* out, float scale) {
  const int D = p->cfg.head_dim;
  char* ws = (char*)workspace;
  PrefillParams a{};
  a.pool = (const uint16_t*)p->cfg.base + (uint64_t)layer * ((uint64_t)2 * p->cfg.num_kv_heads * 16 * D);
  a.work = (const WorkItem*)(ws + p->pf.off_work);
  a.tiles = (const int32_t*)(ws + p->pf.off_tiles);
  a.tile_base = (const int32_t*)(ws + p->pf.off_tile_base);
  a.order = (const int32_t*)(ws + p->pf.off_order);
  a.merge_tiles = (const int32_t*)(ws + p->pf.off_merge_tiles);
  a.q = (const uint16_t*)q;
  a.table = table;
  a.part_acc = (float*)(ws + p->pf.off_acc);
  a.part_ml = (float*)(ws + p->pf.off_ml);
  a.out = (float*)out;
  a.err = (uint32_t*)ws;
  a.block_elems = p->block_elems;
  a.v_off = (uint32_t)(p->cfg.num_kv_heads * 16 * D);
  a.max_blk = max_blk;
  a.Hq = p->cfg.num_q_heads;
  a.Hkv = p->cfg.num_kv_heads;
  a.G = p->G;
  a.gp_shift = p->pf.gp_shift;
  a.NB = p->cfg.num_blocks;
  a.scale_log2 = (scale != 0.f ? scale : 1.0f / std::sqrt((float)D)) * 1.4426950408889634f;
  return a;
}

static int pf_launch_slice(vkv_pool* p, int32_t layer, int32_t slice, const void* q, const int32_t* table,
                           int32_t max_blk, void* workspace, void* out, float scale, hipStream_t st) {
  PrefillParams a = pf_params(p, layer, q, table, max_blk, workspace, out, scale);
  a.item_first = p->pf.slice_start[slice];
  const int32_t count = p->pf.slice_start[slice + 1] - a.item_first;
  ProfKernel prof(p, VKV_PROF_PREFILL, slice);
  prof.launch(paged_prefill_attn_slice_kernel<128>, dim3((unsigned)count), dim3(256), st, a);
  VKV_HIP(hipGetLastError());
  return VKV_OK;
}

// merge step `step` covers tiles [merge_start[step], merge_start[step + 1])
static int pf_launch_merge(vkv_pool* p, int32_t step, void* workspace, void* out, hipStream_t st) {
  PrefillParams a = pf_params(p, 0, workspace, nullptr, 0, workspace, out, 0.f);
  a.item_first = p->pf.merge_start[step];
  const int32_t n_tiles = p->pf.merge_start[step + 1] - a.item_first;
  if (n_tiles == 0) return VKV_OK;   // no tile of this plan was split
  ProfScope prof(p, VKV_PROF_PREFILL_MERGE, step, st);
  hipLaunchKernelGGL(prefill_merge_kernel<128>, dim3((unsigned)(n_tiles * p->cfg.num_kv_heads * (kTileColumns / kMergeCols))),
                     dim3(256), 0, st, a);
  VKV_HIP(hipGetLastError());
  return VKV_OK;
}

}  // namespace vkv

using namespace vkv;

extern "C" {

int kv_prefill_plan(vkv_pool* p, const int32_t* ctx, const int32_t* q_len, int32_t S, uint64_t slice_bytes,
                    int32_t chunk_tokens, vkv_prefill_plan_info* info) {
  if (!p || !ctx || !q_len || S < 1) { set_error("kv_prefill_plan: bad argument"); return VKV_E_INVAL; }
  if (chunk_tokens < kGroupTokens || chunk_tokens % kGroupTokens || chunk_tokens > kMaxPrefillChunkTokens) {
    set_error("kv_prefill_plan: chunk_tokens must be a multiple of %d in [%d, %d]", kGroupTokens, kGroupTokens,
              kMaxPrefillChunkTokens);
    return VKV_E_INVAL;
  }
  const int Hkv = p->cfg.num_kv_heads, D = p->cfg.head_dim, B = p->cfg.block_tokens, G = p->G;
  if (D != 128) { set_error("kv_prefill_plan: prefill supports head_dim 128 only (pool has %d)", D); return VKV_E_INVAL; }
  int gp_shift = 0;
  while ((1 << gp_shift) < G) ++gp_shift;
  const int QP = kTileColumns >> gp_shift;   // positions per tile
  vkv_pool::PrefillPlan pl;
  pl.gp_shift = gp_shift;
  pl.tile_positions = QP;
  pl.num_seqs = S;
  int64_t row = 0;
  double flops = 0.0;
  uint64_t total = 0, max_slice = 0;
  for (int32_t s = 0; s < S; ++s) {
    if (q_len[s] < 1 || ctx[s] < q_len[s]) {
      set_error("kv_prefill_plan: sequence %d needs 1 <= q_len (%d) <= context length (%d)", s, q_len[s], ctx[s]);
      return VKV_E_INVAL;
    }
    pl.max_ctx_blocks = std::max(pl.max_ctx_blocks, (ctx[s] + B - 1) / B);
    const int32_t q0 = ctx[s] - q_len[s];
    for (int32_t t = 0; t * QP < q_len[s]; ++t) {
      const int32_t n_pos = std::min(QP, q_len[s] - t * QP), pos0 = q0 + t * QP, visible = pos0 + n_pos;
      const int32_t tile = (int32_t)pl.tile_base.size();
      pl.tiles.insert(pl.tiles.end(), {s, (int32_t)(row + (int64_t)t * QP), pos0, n_pos});
      pl.tile_base.push_back((int32_t)pl.work.size());
      for (int32_t first = 0; first < visible; first += chunk_tokens) {
        const int32_t nt = std::min(chunk_tokens, visible - first);
        for (int32_t h = 0; h < Hkv; ++h) pl.work.push_back(WorkItem{tile, h, first / B, nt});
      }
      if (pl.work.size() > 0x7FFFFF00u) { set_error("kv_prefill_plan: too many work items"); return VKV_E_INVAL; }
      for (int32_t i = 0; i < n_pos; ++i) flops += 4.0 * D * p->cfg.num_q_heads * (double)(pos0 + i + 1);
    }
    row += q_len[s];
  }
  if (row > 0x7FFFFFF0ll) { set_error("kv_prefill_plan: too many query rows"); return VKV_E_INVAL; }
  pl.total_q = (int32_t)row;
  pl.tile_base.push_back((int32_t)pl.work.size());
  const uint64_t token_bytes = (uint64_t)2 * D * 2;
  pl.slice_start.push_back(0);
  uint64_t acc = 0;
  for (size_t i = 0; i < pl.work.size(); ++i) {
    const uint64_t b = (uint64_t)pl.work[i].n_tokens * token_bytes;
    if ((int32_t)i > pl.slice_start.back() && acc + b > slice_bytes) {
      max_slice = std::max(max_slice, acc);
      pl.slice_start.push_back((int32_t)i);
      acc = 0;
    }
    acc += b;
    total += b;
  }
  max_slice = std::max(max_slice, acc);
  pl.slice_start.push_back((int32_t)pl.work.size());
  const uint64_t n_items = pl.work.size(), n_tiles = pl.tile_base.size() - 1;
  // The merge of split tiles is cut into steps as well, so that it cannot hold up a yield: a step
  // is a run of split tiles whose partial results and outputs amount to at most slice_bytes / 2.
  {
    const uint64_t tile_part = (uint64_t)kTileColumns * D * 4 * Hkv, bound = std::max<uint64_t>(slice_bytes / 2, tile_part);
    uint64_t acc_b = 0;
    pl.merge_start.push_back(0);
    for (size_t t = 0; t + 1 < pl.tile_base.size(); ++t) {
      const uint64_t nch = (uint64_t)(pl.tile_base[t + 1] - pl.tile_base[t]) / Hkv;
      if (nch <= 1) continue;
      const uint64_t b = (nch + 1) * tile_part;
      if (acc_b + b > bound && acc_b > 0) {
        pl.merge_start.push_back((int32_t)pl.merge_tiles.size());
        acc_b = 0;
      }
      pl.merge_tiles.push_back((int32_t)t);
      acc_b += b;
    }
    pl.merge_start.push_back((int32_t)pl.merge_tiles.size());
  }
  pl.off_work = 256;
  pl.off_tiles = pl.off_work + n_items * sizeof(WorkItem);
  pl.off_tile_base = pl.off_tiles + n_tiles * 16;
  pl.off_order = pl.off_tile_base + (n_tiles + 1) * 4;
  pl.off_merge_tiles = pl.off_order + n_items * 4;
  pl.upload_bytes = pl.off_merge_tiles + pl.merge_tiles.size() * 4;
  // Workgroups start in grid order: the longest items of a slice go first so that the short ones fill
  // the tail.  Results are stored by item id, so the order is invisible outside the kernel.
  pl.order.resize(n_items);
  for (size_t i = 0; i < n_items; ++i) pl.order[i] = (int32_t)i;
  for (size_t sl = 0; sl + 1 < pl.slice_start.size(); ++sl)
    std::stable_sort(pl.order.begin() + pl.slice_start[sl], pl.order.begin() + pl.slice_start[sl + 1],
                     [&](int32_t a, int32_t b) { return pl.work[a].n_tokens > pl.work[b].n_tokens; });
  pl.off_ml = align_up(pl.upload_bytes, 256);
  pl.off_acc = align_up(pl.off_ml + n_items * kTileColumns * 2 * 4, 256);
  pl.total = align_up(pl.off_acc + n_items * kTileColumns * (uint64_t)D * 4, 256);
  pl.has_plan = true;
  pl.gen = p->pf.gen + 1;
  p->pf = std::move(pl);
  if (info) {
    info->n_items = (int32_t)n_items;
    info->n_slices = (int32_t)p->pf.slice_start.size() - 1;
    info->n_tiles = (int32_t)n_tiles;
    info->tile_positions = QP;
    info->total_q = p->pf.total_q;
    info->n_merge_steps = (int32_t)p->pf.merge_start.size() - 1;
    info->workspace_bytes = p->pf.total;
    info->kv_bytes_per_layer = total;
    info->max_slice_kv_bytes = max_slice;
    info->flops_per_layer = flops;
  }
  return VKV_OK;
}

int kv_prefill_plan_read(vkv_pool* p, int32_t* work_out, int32_t* slice_start_out, int32_t* tiles_out,
                         int32_t* tile_base_out) {
  if (!p) { set_error("kv_prefill_plan_read: null pool"); return VKV_E_INVAL; }
  if (!p->pf.has_plan) { set_error("kv_prefill_plan_read: no plan"); return VKV_E_STATE; }
  if (work_out) std::memcpy(work_out, p->pf.work.data(), p->pf.work.size() * sizeof(WorkItem));
  if (slice_start_out) std::memcpy(slice_start_out, p->pf.slice_start.data(), p->pf.slice_start.size() * 4);
  if (tiles_out) std::memcpy(tiles_out, p->pf.tiles.data(), p->pf.tiles.size() * 4);
  if (tile_base_out) std::memcpy(tile_base_out, p->pf.tile_base.data(), p->pf.tile_base.size() * 4);
  return VKV_OK;
}

int kv_prefill_bind(vkv_pool* p, void* workspace, uint64_t workspace_bytes, void* stream) {
  if (!p) { set_error("kv_prefill_bind: null pool"); return VKV_E_INVAL; }
  if (p->broken) { set_error("kv_prefill_bind: pool unusable after a HIP failure"); return VKV_E_HIP; }
  if (!p->pf.has_plan) { set_error("kv_prefill_bind: no plan"); return VKV_E_STATE; }
  if (!workspace || (uintptr_t)workspace % 256 || workspace_bytes < p->pf.total) {
    set_error("kv_prefill_bind: workspace must be 256-byte aligned and hold %llu bytes", (unsigned long long)p->pf.total);
    return VKV_E_INVAL;
  }
  int st = ensure_stage(p, p->pf.upload_bytes);
  if (st != VKV_OK) return st;
  char* h = (char*)p->stage;
  std::memset(h, 0, 256);
  std::memcpy(h + p->pf.off_work, p->pf.work.data(), p->pf.work.size() * sizeof(WorkItem));
  std::memcpy(h + p->pf.off_tiles, p->pf.tiles.data(), p->pf.tiles.size() * 4);
  std::memcpy(h + p->pf.off_tile_base, p->pf.tile_base.data(), p->pf.tile_base.size() * 4);
  std::memcpy(h + p->pf.off_order, p->pf.order.data(), p->pf.order.size() * 4);
  std::memcpy(h + p->pf.off_merge_tiles, p->pf.merge_tiles.data(), p->pf.merge_tiles.size() * 4);
  VKV_HIP(hipMemcpyAsync(workspace, h, p->pf.upload_bytes, hipMemcpyHostToDevice, (hipStream_t)stream));
  VKV_HIP(hipEventRecord(p->stage_ev, (hipStream_t)stream));
  p->stage_inflight = true;
  p->pf.bound_ws = workspace;
  p->pf.bound_gen = p->pf.gen;
  return VKV_OK;
}

int paged_prefill_attn_slice(vkv_pool* p, int32_t layer, int32_t slice, const void* q, const int32_t* table,
                             int32_t max_blk, void* workspace, void* out, float scale, void* stream) {
  int st = pf_check_args(p, layer, q, table, max_blk, workspace, out, "paged_prefill_attn_slice");
  if (st != VKV_OK) return st;
  if (slice < 0 || slice >= (int32_t)p->pf.slice_start.size() - 1) {
    set_error("paged_prefill_attn_slice: slice %d out of range [0,%d)", slice, (int)p->pf.slice_start.size() - 1);
    return VKV_E_INVAL;
  }
  return pf_launch_slice(p, layer, slice, q, table, max_blk, workspace, out, scale, (hipStream_t)stream);
}

int kv_prefill_merge(vkv_pool* p, int32_t step, void* workspace, void* out, void* stream) {
  int st = pf_check_bound(p, workspace, "kv_prefill_merge");
  if (st != VKV_OK) return st;
  if (!out) { set_error("kv_prefill_merge: null output"); return VKV_E_INVAL; }
  if (step < 0 || step >= (int32_t)p->pf.merge_start.size() - 1) {
    set_error("kv_prefill_merge: step %d out of range [0,%d)", step, (int)p->pf.merge_start.size() - 1);
    return VKV_E_INVAL;
  }
  return pf_launch_merge(p, step, workspace, out, (hipStream_t)stream);
}

int kv_prefill_run_layer(vkv_pool* p, int32_t layer, int32_t* cursor, const void* q, const int32_t* table,
                         int32_t max_blk, void* workspace, void* out, float scale, int32_t max_inflight,
                         void* stream) {
  int st = pf_check_args(p, layer, q, table, max_blk, workspace, out, "kv_prefill_run_layer");
  if (st != VKV_OK) return st;
  hipStream_t hs = (hipStream_t)stream;
  return run_slices(p, cursor, (int32_t)p->pf.slice_start.size() - 1, max_inflight, hs, "kv_prefill_run_layer",
                    [&](int32_t s, hipStream_t on) {
                      return pf_launch_slice(p, layer, s, q, table, max_blk, workspace, out, scale, on);
                    },
                    (int32_t)p->pf.merge_start.size() - 1,
                    [&](int32_t step) { return pf_launch_merge(p, step, workspace, out, hs); }, false);
}

int kv_prefill_check(vkv_pool* p, void* workspace, void* stream) {
  int st = pf_check_bound(p, workspace, "kv_prefill_check");
  if (st != VKV_OK) return st;
  VKV_HIP(hipStreamSynchronize((hipStream_t)stream));
  uint32_t flag = 0;
  VKV_HIP(hipMemcpy(&flag, workspace, 4, hipMemcpyDeviceToHost));
  if (flag) { set_error("kv_prefill_check: a slice met a block-table entry outside the pool"); return VKV_E_STATE; }
  return VKV_OK;
}

}  // extern "C"
