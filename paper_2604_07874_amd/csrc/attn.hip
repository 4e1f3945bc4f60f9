// Preemptible decode attention over the paged bf16 KV pool.
//
// One layer's attention is cut into work items (sequence, kv head, chunk of tokens) and
// the items into slices of bounded KV bytes; each slice is one launch, so a yield lands
// at a slice boundary (the sub-millisecond bound of paper Section 2.3, Challenge 1 and
// Section 4.1, met without a driver).  The kernel is HBM-bound: it reads every K and V
// byte of its tokens once; the MFMA units do the GQA q.K and p.V tiles.
//
// Kernel shape (wave64, gfx950):
//   workgroup = 4 waves = one work item; wave w takes the 32-token groups w, w+4, ...
//   Per group a wave issues 16 coalesced 16-byte-per-lane loads (K and V rows of two
//   blocks): lane (c = lane%16, kg = lane/16) gets bytes [16c,16c+16) of rows kg, 4+kg,
//   8+kg, 12+kg of each block.
//   K rows go through a per-wave LDS tile to reach the A-operand layout of
//   v_mfma_f32_16x16x32_bf16 (row = token, 8 consecutive d per lane); the B operand is q,
//   one query head per column, columns >= G zero.
//   Scores come back with column = query head = lane%16 and rows kg*4..kg*4+3; tokens are
//   assigned to rows so that row kg*4+r is the token the same lane group loaded as its
//   r-th V row.  The V registers therefore feed the second MFMA (out^T = V^T . P^T)
//   straight from the loads after an in-register 16-bit transpose, with no LDS traffic:
//   lane c owns output dims {c*D/16 + dt}.
//   Softmax statistics are per lane (= per query head): running max m (log2 units), sum l,
//   and the accumulator is rescaled when m grows.  l is summed from the bf16-rounded
//   weights that enter the MFMA, so the result is an exact convex combination of V rows.
//   The block ids of the item sit in two VGPRs (one table entry per lane) and are read
//   with v_readlane, so no load sits between two groups' K/V fetches.
//   Merge: an item that covers its whole sequence writes the output directly.  Otherwise
//   it writes (max, sum, weighted V sum) to the workspace and bumps a per-(sequence, kv
//   head) counter; the workgroup that brings the counter to the chunk count merges all
//   chunks in chunk order (so the bits do not depend on which one arrives last), writes
//   the output and zeroes the counter.  The counters live in the workspace, so this
//   works across slices and across a yield.
#include "vkv_internal.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <functional>

namespace vkv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

struct AttnParams {
  const uint16_t* pool;      // pool base + layer offset (elements)
  const WorkItem* work;      // device; in launch order: inside a slice, items by falling token count
  const uint16_t* q;         // [S][Hq][D]
  const int32_t* table;      // [rows][max_blk]
  float* part_acc;           // [n_items][G][D]
  float* part_ml;            // [n_items][G][2]
  const int32_t* seq_base;   // [S+1] first item of each sequence
  int32_t* done;             // [S][Hkv] chunks finished in the current layer
  float* out;                // [S][Hq][D]
  uint32_t* err;             // workspace header word 0
  uint64_t block_elems;
  uint32_t v_off;            // elements from a block's K plane to its V plane (one layer)
  int32_t item_first;
  int32_t max_blk;
  int32_t Hq, Hkv, G, NB;
  int32_t chunk_blocks;      // blocks per full chunk (chunk_tokens / 16)
  float scale_log2;          // softmax scale * log2(e)
};

template <int D> struct LdVec;
template <> struct LdVec<128> { using type = u32x4; };
template <> struct LdVec<64> { using type = u32x2; };

// device-scope relaxed atomic accesses: coherent across the whole GPU without cache maintenance
__device__ __forceinline__ void st_dev(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_dev(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// word j of a lane-row register as 32 bits (two bf16)
__device__ __forceinline__ uint32_t word_of(const u32x4& v, int j) { return v[j]; }
__device__ __forceinline__ uint32_t word_of(const u32x2& v, int j) { return v[j]; }

template <int D>
__global__ __launch_bounds__(256, 2) void paged_decode_attn_slice_kernel(const AttnParams p) {
  using ldvec = typename LdVec<D>::type;
  constexpr int EPL = D / 16;          // bf16 per lane per row (8 or 4)
  constexpr int KS = D / 32;           // MFMA k-steps of the score tile
  constexpr int RS = D * 2 + 16;       // LDS row stride in bytes (padded against bank conflicts)
  constexpr int TILE = 32 * RS;        // one wave's K tile
  constexpr float NEG_INF = -INFINITY;

  __shared__ __attribute__((aligned(16))) unsigned char lds[4 * TILE];
  __shared__ float sm_m[4][16], sm_l[4][16];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c16 = lane & 15, kg = lane >> 4;

  const WorkItem it = p.work[p.item_first + blockIdx.x];   // workgroups start in grid order: longest items first
  const int ntok = it.n_tokens;
  const int ngroups = (ntok + kGroupTokens - 1) / kGroupTokens;
  const int G = p.G;

  // B operand of the score MFMA: column = query head, k index kg*8+j <-> d = 32*ks + 8*kg + j
  bf16x8 qb[KS];
  {
    const bool valid = c16 < G;
    const uint16_t* qrow = p.q + ((size_t)it.seq * p.Hq + (size_t)it.kv_head * G + (valid ? c16 : 0)) * D;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (valid) v = *reinterpret_cast<const u32x4*>(qrow + ks * 32 + kg * 8);
      qb[ks] = __builtin_bit_cast(bf16x8, v);
    }
  }

  const int32_t* trow = p.table + (size_t)it.seq * p.max_blk + it.first_block;
  const uint16_t* kplane = p.pool + (size_t)it.kv_head * (16 * D);
  unsigned char* tile = lds + wave * TILE;

  // block ids of this item: lane j holds entries j and 64+j (chunk_tokens <= 2048)
  const int nblk_item = (ntok + 15) >> 4;
  const int32_t tb0 = lane < nblk_item ? trow[lane] : -1;
  const int32_t tb1 = 64 + lane < nblk_item ? trow[64 + lane] : -1;

  f32x4 acc[EPL];
#pragma unroll
  for (int dt = 0; dt < EPL; ++dt) acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = NEG_INF, l_run = 0.f;

  ldvec kr[8], vr[8];   // [block b of the group][row slot r]: row 4r+kg of block b

  auto issue = [&](int grp) {
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int bi = grp * 2 + b;
      const bool have = bi < nblk_item;
      const int32_t blk = bi < 64 ? __builtin_amdgcn_readlane(tb0, bi & 63) : __builtin_amdgcn_readlane(tb1, bi & 63);
      if (blk < 0 || blk >= p.NB) {
        if (have && lane == 0) atomicOr(p.err, 1u);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          kr[b * 4 + r] = ldvec{};
          vr[b * 4 + r] = ldvec{};
        }
      } else {
        const ldvec* ks = reinterpret_cast<const ldvec*>(kplane + (size_t)blk * p.block_elems);
        const ldvec* vs = reinterpret_cast<const ldvec*>(kplane + (size_t)blk * p.block_elems + p.v_off);
#pragma unroll
        for (int r = 0; r < 4; ++r) kr[b * 4 + r] = __builtin_nontemporal_load(ks + r * 64 + lane);   // read once
#pragma unroll
        for (int r = 0; r < 4; ++r) vr[b * 4 + r] = __builtin_nontemporal_load(vs + r * 64 + lane);
      }
    }
  };

  int grp = wave;
  if (grp < ngroups) issue(grp);

  for (; grp < ngroups; grp += 4) {
    const int tok0 = grp * kGroupTokens;
    const bool tail = tok0 + kGroupTokens > ntok;

    // K rows -> LDS tile, row index = 16b + 4r + kg, 16-byte column c16
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        *reinterpret_cast<ldvec*>(tile + (b * 16 + 4 * r + kg) * RS + c16 * (EPL * 2)) = kr[b * 4 + r];

    // V rows past the end of the sequence may hold anything (NaN included): zero them
    if (tail) {
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (tok0 + b * 16 + 4 * r + kg >= ntok) vr[b * 4 + r] = ldvec{};
    }

    // A operands of the second MFMA: va[dt] = element dt of each of the lane's 8 V rows
    bf16x8 va[EPL];
#pragma unroll
    for (int dt = 0; dt < EPL; ++dt) {
      u32x4 w;
      const uint32_t sel = (dt & 1) ? 0x07060302u : 0x05040100u;   // high or low halves of (hi=src0, lo=src1)
#pragma unroll
      for (int pr = 0; pr < 4; ++pr)
        w[pr] = __builtin_amdgcn_perm(word_of(vr[2 * pr + 1], dt >> 1), word_of(vr[2 * pr], dt >> 1), sel);
      va[dt] = __builtin_bit_cast(bf16x8, w);
    }

    const int next = grp + 4;
    if (next < ngroups) issue(next);

    // LDS operations of one wave execute in order; keep the compiler from reordering them
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // scores: tile b, MFMA row i <-> token 4*(i%4) + i/4 of block b
    f32x4 sc[2];
    const int trow_lds = 4 * (c16 & 3) + (c16 >> 2);
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      sc[b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const u32x4 a = *reinterpret_cast<const u32x4*>(tile + (b * 16 + trow_lds) * RS + (ks * 4 + kg) * 16);
        sc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), qb[ks], sc[b], 0, 0, 0);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    // this lane: query head c16, tokens tok0 + 16b + 4r + kg
    float x[8];
    float mx = NEG_INF;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const bool ok = !tail || (tok0 + b * 16 + 4 * r + kg < ntok);
        const float v = ok ? sc[b][r] * p.scale_log2 : NEG_INF;
        x[b * 4 + r] = v;
        mx = fmaxf(mx, v);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);           // finite: every group holds a valid token
    const float alpha = __builtin_exp2f(m_run - m_new);
    bf16x8 pb;
    float psum = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const __bf16 pj = (__bf16)__builtin_exp2f(x[j] - m_new);
      pb[j] = pj;
      psum += (float)pj;
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int dt = 0; dt < EPL; ++dt) {
      acc[dt] *= alpha;
      acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[dt], pb, acc[dt], 0, 0, 0);
    }
  }

  // ---- merge the four waves (each covered a disjoint subset of the item's tokens) ----
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  __syncthreads();   // all waves are done with their K tiles
  float* macc = reinterpret_cast<float*>(lds);   // [4][G][D]
  if (c16 < G) {
#pragma unroll
    for (int dt = 0; dt < EPL; ++dt)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        macc[((size_t)wave * G + c16) * D + (kg * 4 + r) * EPL + dt] = acc[dt][r];
    if (kg == 0) {
      sm_m[wave][c16] = m_run;
      sm_l[wave][c16] = l_run;
    }
  }
  __syncthreads();
  const int base = p.seq_base[it.seq];
  // item id in plan order (sequence, chunk, kv head): partial results are stored under it
  const size_t item = (size_t)base + (size_t)(it.first_block / p.chunk_blocks) * p.Hkv + it.kv_head;
  const int nch = (p.seq_base[it.seq + 1] - base) / p.Hkv;   // chunks of this sequence
  float* orow = p.out + ((size_t)it.seq * p.Hq + (size_t)it.kv_head * G) * D;
  for (int e = threadIdx.x; e < G * D; e += 256) {
    const int g = e / D, d = e - g * D;
    float M = sm_m[0][g];
#pragma unroll
    for (int w = 1; w < 4; ++w) M = fmaxf(M, sm_m[w][g]);
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float wt = __builtin_exp2f(sm_m[w][g] - M);   // 0 for a wave that had no group
      num += wt * macc[((size_t)w * G + g) * D + d];
      den += wt * sm_l[w][g];
    }
    if (nch == 1) {
      orow[e] = num / den;
    } else {
      st_dev(&p.part_acc[(item * G + g) * D + d], num);
      if (d == 0) {
        st_dev(&p.part_ml[(item * G + g) * 2 + 0], M);
        st_dev(&p.part_ml[(item * G + g) * 2 + 1], den);
      }
    }
  }
  if (nch == 1) return;

  // Publish the partial result, then count this chunk as done.  The partial results and the
  // counter are only ever touched with device-scope atomic accesses, which are performed at
  // the device's coherence point (not in the per-XCD L2), so no cache write-back or
  // invalidation is needed: each wave waits until its stores are acknowledged, the barrier
  // collects the waves, then thread 0 bumps the counter.
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();
  __shared__ int sm_last;
  int32_t* done = p.done + (size_t)it.seq * p.Hkv + it.kv_head;
  if (threadIdx.x == 0)
    sm_last = __hip_atomic_fetch_add(done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == nch - 1;
  __syncthreads();
  if (!sm_last) return;
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");

  // Last chunk of this (sequence, kv head): merge all chunks, in chunk order.
  // Stage every chunk's (max, sum) in LDS first so the loads below are independent.
  float* cm = reinterpret_cast<float*>(lds);       // [nch][G]
  float* cl = cm + (size_t)nch * G;                 // [nch][G]
  for (int i = threadIdx.x; i < nch * G; i += 256) {
    const int c = i / G, g = i - c * G;
    const size_t ig = ((size_t)base + (size_t)c * p.Hkv + it.kv_head) * G + g;
    cm[i] = ld_dev(&p.part_ml[ig * 2]);
    cl[i] = ld_dev(&p.part_ml[ig * 2 + 1]);
  }
  __syncthreads();
  for (int e = threadIdx.x; e < G * D; e += 256) {
    const int g = e / D, d = e - g * D;
    float M = NEG_INF;
    for (int c = 0; c < nch; ++c) M = fmaxf(M, cm[c * G + g]);
    float num = 0.f, den = 0.f;
    for (int c0 = 0; c0 < nch; c0 += 8) {
      float a[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int c = c0 + j < nch ? c0 + j : nch - 1;
        a[j] = ld_dev(&p.part_acc[(((size_t)base + (size_t)c * p.Hkv + it.kv_head) * G + g) * D + d]);
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (c0 + j < nch) {
          const float wt = __builtin_exp2f(cm[(c0 + j) * G + g] - M);
          num += wt * a[j];
          den += wt * cl[(c0 + j) * G + g];
        }
      }
    }
    orow[e] = num / den;
  }
  if (threadIdx.x == 0) __hip_atomic_store(done, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next layer
}

// ---- host ---------------------------------------------------------------------------

// Yardstick: the memory accesses of the slice kernel without its arithmetic.  Same work items,
// same 4 KiB runs, same 16 loads per wave and group requested one group ahead; the values are
// xor-ed and stored only if they equal one fixed pattern.  What this reads per second is what the
// access pattern allows; the gap to the real kernel is compute, merge and bookkeeping.
template <int D>
__global__ __launch_bounds__(256, 2) void paged_read_probe_kernel(const AttnParams p, u32x4* __restrict__ sink) {
  using ldvec = typename LdVec<D>::type;
  // as much LDS as keeps two workgroups on a compute unit, the slice kernel's own occupancy
  __shared__ uint32_t occupancy_pad[(72 * 1024) / 4];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const WorkItem it = p.work[p.item_first + blockIdx.x];
  const int ntok = it.n_tokens;
  if (ntok < 0) occupancy_pad[threadIdx.x] = (uint32_t)ntok;   // never true; keeps the array allocated
  const int ngroups = (ntok + kGroupTokens - 1) / kGroupTokens;
  const int32_t* trow = p.table + (size_t)it.seq * p.max_blk + it.first_block;
  const uint16_t* kplane = p.pool + (size_t)it.kv_head * (16 * D);
  const int nblk_item = (ntok + 15) >> 4;
  const int32_t tb0 = lane < nblk_item ? trow[lane] : -1;
  const int32_t tb1 = 64 + lane < nblk_item ? trow[64 + lane] : -1;
  ldvec r[16];
  auto issue = [&](int grp) {
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int bi = grp * 2 + b;
      const int32_t blk = bi < 64 ? __builtin_amdgcn_readlane(tb0, bi & 63) : __builtin_amdgcn_readlane(tb1, bi & 63);
      if (blk < 0 || blk >= p.NB) {
#pragma unroll
        for (int i = 0; i < 8; ++i) r[b * 8 + i] = ldvec{};
      } else {
        const ldvec* ks = reinterpret_cast<const ldvec*>(kplane + (size_t)blk * p.block_elems);
        const ldvec* vs = reinterpret_cast<const ldvec*>(kplane + (size_t)blk * p.block_elems + p.v_off);
#pragma unroll
        for (int i = 0; i < 4; ++i) r[b * 8 + i] = __builtin_nontemporal_load(ks + i * 64 + lane);
#pragma unroll
        for (int i = 0; i < 4; ++i) r[b * 8 + 4 + i] = __builtin_nontemporal_load(vs + i * 64 + lane);
      }
    }
  };
  ldvec acc{};
  int grp = wave;
  if (grp < ngroups) issue(grp);
  for (; grp < ngroups; grp += 4) {
    ldvec x{};
#pragma unroll
    for (int i = 0; i < 16; ++i) x ^= r[i];
    if (grp + 4 < ngroups) issue(grp + 4);
    acc ^= x;
  }
  if (acc[0] == 0x9E3779B9u && acc[1] == 0x7F4A7C15u) sink[threadIdx.x & 15] = u32x4{acc[0], acc[1], 0u, 0u};
}

static int check_bound(vkv_pool* p, const void* workspace, const char* who) {
  if (!p) { set_error("%s: null pool", who); return VKV_E_INVAL; }
  if (p->broken) { set_error("%s: pool unusable after a HIP failure", who); return VKV_E_HIP; }
  if (!p->has_plan) { set_error("%s: no plan; call kv_attn_plan first", who); return VKV_E_STATE; }
  if (!workspace || workspace != p->bound_ws || p->bound_gen != p->plan_gen) {
    set_error("%s: workspace is not bound to the current plan; call kv_attn_bind", who);
    return VKV_E_STATE;
  }
  return VKV_OK;
}

static int launch_slice(vkv_pool* p, int32_t layer, int32_t slice, const void* q, const int32_t* table,
                        int32_t max_blk, void* workspace, void* out, float scale, hipStream_t st) {
  const int32_t first = p->slice_start[slice], count = p->slice_start[slice + 1] - first;
  const int D = p->cfg.head_dim;
  char* ws = (char*)workspace;
  AttnParams a;
  const uint64_t layer_elems = (uint64_t)2 * p->cfg.num_kv_heads * 16 * D;
  a.pool = (const uint16_t*)p->cfg.base + (uint64_t)layer * layer_elems;
  a.work = (const WorkItem*)(ws + p->ws.work);
  a.q = (const uint16_t*)q;
  a.table = table;
  a.part_acc = (float*)(ws + p->ws.part_acc);
  a.part_ml = (float*)(ws + p->ws.part_ml);
  a.seq_base = (const int32_t*)(ws + p->ws.seq_base);
  a.chunk_blocks = p->chunk_tokens / p->cfg.block_tokens;
  a.done = (int32_t*)(ws + p->ws.done);
  a.out = (float*)out;
  a.err = (uint32_t*)(ws + p->ws.header);
  a.block_elems = p->block_elems;
  a.v_off = (uint32_t)(p->cfg.num_kv_heads * 16 * D);
  a.item_first = first;
  a.max_blk = max_blk;
  a.Hq = p->cfg.num_q_heads;
  a.Hkv = p->cfg.num_kv_heads;
  a.G = p->G;
  a.NB = p->cfg.num_blocks;
  a.scale_log2 = (scale != 0.f ? scale : 1.0f / std::sqrt((float)D)) * 1.4426950408889634f;
  ProfScope prof(p, VKV_PROF_SLICE, slice, st);
  if (D == 128)
    hipLaunchKernelGGL(paged_decode_attn_slice_kernel<128>, dim3((unsigned)count), dim3(256), 0, st, a);
  else
    hipLaunchKernelGGL(paged_decode_attn_slice_kernel<64>, dim3((unsigned)count), dim3(256), 0, st, a);
  VKV_HIP(hipGetLastError());
  return VKV_OK;
}

static int check_slice_args(vkv_pool* p, int32_t layer, const void* q, const int32_t* table, int32_t max_blk,
                            void* workspace, void* out, const char* who) {
  int st = check_bound(p, workspace, who);
  if (st != VKV_OK) return st;
  if (!p->cfg.base) { set_error("%s: pool has no device memory", who); return VKV_E_INVAL; }
  if (layer < 0 || layer >= p->cfg.num_layers) { set_error("%s: layer %d out of range", who, layer); return VKV_E_INVAL; }
  if (!q || !table || !out || (uintptr_t)q % 16) {
    set_error("%s: q (16-byte aligned), block_table and out must be given", who);
    return VKV_E_INVAL;
  }
  if (max_blk < p->max_ctx_blocks) {
    set_error("%s: block table has %d columns, the plan needs %d", who, max_blk, p->max_ctx_blocks);
    return VKV_E_INVAL;
  }
  return VKV_OK;
}

// Slice scheduler shared by decode and prefill: issues steps *cursor .. n_slices + n_tail - 1
// (slices through `launch`, then n_tail follow-up steps through `tail`, all on the caller's
// stream), keeping at most max_inflight launches unfinished; the ring of events persists across
// calls.  Stops at a step boundary when the yield flag is set.
// With overlap on, odd slices go to a second stream the pool owns (forked from and joined back
// into the caller's stream inside this call), so the workgroups of the next slice fill the
// compute units the tail of the previous one leaves idle; slices of one layer are independent
// (results are merged through per-item partials), so their order does not matter.
int run_slices(vkv_pool* p, int32_t* cursor, int32_t n_slices, int32_t max_inflight, hipStream_t hs,
               const char* who, const std::function<int(int32_t, hipStream_t)>& launch, int32_t n_tail,
               const std::function<int(int32_t)>& tail) {
  if (!cursor || *cursor < 0 || *cursor > n_slices + n_tail || max_inflight < 1 || max_inflight > kMaxInflight) {
    set_error("%s: bad cursor or max_inflight", who);
    return VKV_E_INVAL;
  }
  int st = VKV_OK;
  for (int i = 0; i < max_inflight; ++i)
    if (!p->inflight_ev[i]) VKV_HIP(hipEventCreateWithFlags(&p->inflight_ev[i], hipEventDisableTiming));
  auto drain = [&]() -> int {
    for (; p->inflight_count > 0; --p->inflight_count, p->inflight_head = (p->inflight_head + 1) % p->inflight_cap)
      VKV_HIP(hipEventSynchronize(p->inflight_ev[p->inflight_head]));
    p->inflight_head = 0;
    return VKV_OK;
  };
  if (p->inflight_cap != max_inflight) {
    st = drain();
    if (st != VKV_OK) return st;
    p->inflight_cap = max_inflight;
  }
  // one more launch may be enqueued once fewer than max_inflight are unfinished
  auto admit = [&]() -> int {
    if (p->inflight_count == max_inflight) {
      VKV_HIP(hipEventSynchronize(p->inflight_ev[p->inflight_head]));
      p->inflight_head = (p->inflight_head + 1) % max_inflight;
      --p->inflight_count;
    }
    return VKV_OK;
  };
  auto track = [&](hipStream_t on) -> int {
    VKV_HIP(hipEventRecord(p->inflight_ev[(p->inflight_head + p->inflight_count) % max_inflight], on));
    ++p->inflight_count;
    return VKV_OK;
  };
  const bool two = p->overlap && p->aux_stream && max_inflight >= 2 && n_slices - *cursor >= 2;
  bool aux_used = false;
  if (two) {
    // the second stream starts after everything the caller has enqueued so far (q, tables, the plan upload)
    VKV_HIP(hipEventRecord(p->fork_ev, hs));
    VKV_HIP(hipStreamWaitEvent(p->aux_stream, p->fork_ev, 0));
  }
  // later work on the caller's stream (the merge, the next layer) waits for the second stream's slices
  auto join = [&]() -> int {
    if (aux_used) {
      VKV_HIP(hipEventRecord(p->join_ev, p->aux_stream));
      VKV_HIP(hipStreamWaitEvent(hs, p->join_ev, 0));
      aux_used = false;
    }
    return VKV_OK;
  };
  for (int32_t s = *cursor; s < n_slices; ++s) {
    if (p->yield_flag.load(std::memory_order_acquire)) {
      st = drain();
      if (st != VKV_OK) return st;
      if ((st = join()) != VKV_OK) return st;
      *cursor = s;
      return VKV_YIELDED;
    }
    const hipStream_t on = (two && (s & 1)) ? p->aux_stream : hs;
    if ((st = admit()) != VKV_OK) return st;
    if ((st = launch(s, on)) != VKV_OK) return st;
    if ((st = track(on)) != VKV_OK) return st;
    if (on != hs) aux_used = true;
  }
  if ((st = join()) != VKV_OK) return st;
  for (int32_t t = std::max(*cursor, n_slices) - n_slices; t < n_tail; ++t) {
    if (p->yield_flag.load(std::memory_order_acquire)) {
      st = drain();
      if (st != VKV_OK) return st;
      *cursor = n_slices + t;
      return VKV_YIELDED;
    }
    if ((st = admit()) != VKV_OK) return st;
    if ((st = tail(t)) != VKV_OK) return st;
    if ((st = track(hs)) != VKV_OK) return st;
  }
  *cursor = n_slices + n_tail;
  return VKV_OK;
}

}  // namespace vkv

using namespace vkv;

extern "C" {

int kv_attn_plan(vkv_pool* p, const int32_t* ctx, int32_t S, uint64_t slice_bytes, int32_t chunk_tokens,
                 vkv_attn_plan_info* info) {
  if (!p || !ctx || S < 1) { set_error("kv_attn_plan: bad argument"); return VKV_E_INVAL; }
  if (chunk_tokens < kGroupTokens || chunk_tokens % kGroupTokens || chunk_tokens > kMaxChunkTokens) {
    set_error("kv_attn_plan: chunk_tokens must be a multiple of %d in [%d, %d]", kGroupTokens, kGroupTokens,
              kMaxChunkTokens);
    return VKV_E_INVAL;
  }
  const int Hkv = p->cfg.num_kv_heads, D = p->cfg.head_dim, B = p->cfg.block_tokens;
  int64_t n_items = 0;
  int32_t max_blocks = 0;
  for (int32_t s = 0; s < S; ++s) {
    if (ctx[s] < 1) { set_error("kv_attn_plan: sequence %d has context length %d (< 1)", s, ctx[s]); return VKV_E_INVAL; }
    n_items += (int64_t)((ctx[s] + chunk_tokens - 1) / chunk_tokens) * Hkv;
    max_blocks = std::max(max_blocks, (ctx[s] + B - 1) / B);
  }
  if (n_items > 0x7FFFFFF0ll) { set_error("kv_attn_plan: too many work items"); return VKV_E_INVAL; }
  {
    // the merge stages (max, sum) of all chunks of one sequence in LDS
    const int64_t max_chunks = ((int64_t)max_blocks * B + chunk_tokens - 1) / chunk_tokens;
    if (max_chunks * p->G * 8 > kMergeLdsBytes) {
      set_error("kv_attn_plan: %lld chunks per sequence is too many for group size %d; raise chunk_tokens",
                (long long)max_chunks, p->G);
      return VKV_E_INVAL;
    }
  }
  std::vector<WorkItem> work;
  std::vector<int32_t> seq_base((size_t)S + 1);
  work.reserve((size_t)n_items);
  for (int32_t s = 0; s < S; ++s) {
    seq_base[s] = (int32_t)work.size();
    for (int32_t first = 0; first < ctx[s]; first += chunk_tokens) {
      const int32_t nt = std::min(chunk_tokens, ctx[s] - first);
      for (int32_t h = 0; h < Hkv; ++h) work.push_back(WorkItem{s, h, first / B, nt});
    }
  }
  seq_base[S] = (int32_t)work.size();
  const uint64_t token_bytes = (uint64_t)2 * D * 2;
  std::vector<int32_t> starts{0};
  uint64_t acc = 0, total = 0, max_slice = 0;
  for (size_t i = 0; i < work.size(); ++i) {
    const uint64_t b = (uint64_t)work[i].n_tokens * token_bytes;
    if ((int32_t)i > starts.back() && acc + b > slice_bytes) {
      max_slice = std::max(max_slice, acc);
      starts.push_back((int32_t)i);
      acc = 0;
    }
    acc += b;
    total += b;
  }
  max_slice = std::max(max_slice, acc);
  starts.push_back((int32_t)work.size());

  // Workgroups start in grid order.  Inside a slice the longest items go first, so the short
  // ones (ragged ends of sequences) fill the tail of the launch; equal items keep the plan's
  // order (the kv heads of one chunk stay neighbours and read one slab together).  Results are
  // stored by item id, so the launch order is invisible outside the kernel.
  std::vector<int32_t> order(work.size());
  for (size_t i = 0; i < order.size(); ++i) order[i] = (int32_t)i;
  for (size_t sl = 0; sl + 1 < starts.size(); ++sl)
    std::stable_sort(order.begin() + starts[sl], order.begin() + starts[sl + 1],
                     [&](int32_t a, int32_t b) { return work[a].n_tokens > work[b].n_tokens; });
  p->order.swap(order);
  p->work.swap(work);
  p->slice_start.swap(starts);
  p->seq_base.swap(seq_base);
  p->num_seqs = S;
  p->chunk_tokens = chunk_tokens;
  p->max_ctx_blocks = max_blocks;
  p->ws = workspace_layout((int64_t)p->work.size(), S, Hkv, p->G, D);
  p->has_plan = true;
  ++p->plan_gen;
  if (info) {
    info->n_items = (int32_t)p->work.size();
    info->n_slices = (int32_t)p->slice_start.size() - 1;
    info->workspace_bytes = p->ws.total;
    info->kv_bytes_per_layer = total;
    info->max_slice_kv_bytes = max_slice;
  }
  return VKV_OK;
}

int kv_attn_plan_read(vkv_pool* p, int32_t* work_out, int32_t* slice_start_out) {
  if (!p) { set_error("kv_attn_plan_read: null pool"); return VKV_E_INVAL; }
  if (!p->has_plan) { set_error("kv_attn_plan_read: no plan"); return VKV_E_STATE; }
  if (work_out) std::memcpy(work_out, p->work.data(), p->work.size() * sizeof(WorkItem));
  if (slice_start_out) std::memcpy(slice_start_out, p->slice_start.data(), p->slice_start.size() * 4);
  return VKV_OK;
}

int kv_attn_bind(vkv_pool* p, void* workspace, uint64_t workspace_bytes, void* stream) {
  if (!p) { set_error("kv_attn_bind: null pool"); return VKV_E_INVAL; }
  if (p->broken) { set_error("kv_attn_bind: pool unusable after a HIP failure"); return VKV_E_HIP; }
  if (!p->has_plan) { set_error("kv_attn_bind: no plan"); return VKV_E_STATE; }
  if (!workspace || (uintptr_t)workspace % 256 || workspace_bytes < p->ws.total) {
    set_error("kv_attn_bind: workspace must be 256-byte aligned and hold %llu bytes",
              (unsigned long long)p->ws.total);
    return VKV_E_INVAL;
  }
  int st = ensure_stage(p, p->ws.upload_bytes);
  if (st != VKV_OK) return st;
  char* h = (char*)p->stage;
  std::memset(h, 0, p->ws.upload_bytes);   // flag word and per-(sequence, kv head) counters start at zero
  WorkItem* hw = (WorkItem*)(h + p->ws.work);
  for (size_t i = 0; i < p->order.size(); ++i) hw[i] = p->work[p->order[i]];   // the device copy is in launch order
  std::memcpy(h + p->ws.seq_base, p->seq_base.data(), p->seq_base.size() * 4);
  VKV_HIP(hipMemcpyAsync(workspace, h, p->ws.upload_bytes, hipMemcpyHostToDevice, (hipStream_t)stream));
  VKV_HIP(hipEventRecord(p->stage_ev, (hipStream_t)stream));
  p->stage_inflight = true;
  p->bound_ws = workspace;
  p->bound_gen = p->plan_gen;
  return VKV_OK;
}

int paged_decode_attn_slice(vkv_pool* p, int32_t layer, int32_t slice, const void* q, const int32_t* table,
                            int32_t max_blk, void* workspace, void* out, float scale, void* stream) {
  int st = check_slice_args(p, layer, q, table, max_blk, workspace, out, "paged_decode_attn_slice");
  if (st != VKV_OK) return st;
  if (slice < 0 || slice >= (int32_t)p->slice_start.size() - 1) {
    set_error("paged_decode_attn_slice: slice %d out of range [0,%d)", slice, (int)p->slice_start.size() - 1);
    return VKV_E_INVAL;
  }
  return launch_slice(p, layer, slice, q, table, max_blk, workspace, out, scale, (hipStream_t)stream);
}

int kv_probe_attn_reads(vkv_pool* p, int32_t layer, int32_t slice, const int32_t* table, int32_t max_blk,
                        void* workspace, void* sink, void* stream) {
  int st = check_slice_args(p, layer, workspace, table, max_blk, workspace, workspace, "kv_probe_attn_reads");
  if (st != VKV_OK) return st;
  if (!sink || (uintptr_t)sink % 16) { set_error("kv_probe_attn_reads: sink must be a 16-byte aligned device pointer"); return VKV_E_INVAL; }
  if (slice < 0 || slice >= (int32_t)p->slice_start.size() - 1) {
    set_error("kv_probe_attn_reads: slice %d out of range [0,%d)", slice, (int)p->slice_start.size() - 1);
    return VKV_E_INVAL;
  }
  const int32_t first = p->slice_start[slice], count = p->slice_start[slice + 1] - first;
  const int D = p->cfg.head_dim;
  AttnParams a{};
  a.pool = (const uint16_t*)p->cfg.base + (uint64_t)layer * ((uint64_t)2 * p->cfg.num_kv_heads * 16 * D);
  a.work = (const WorkItem*)((char*)workspace + p->ws.work);
  a.table = table;
  a.block_elems = p->block_elems;
  a.v_off = (uint32_t)(p->cfg.num_kv_heads * 16 * D);
  a.item_first = first;
  a.max_blk = max_blk;
  a.NB = p->cfg.num_blocks;
  if (D == 128)
    hipLaunchKernelGGL(paged_read_probe_kernel<128>, dim3((unsigned)count), dim3(256), 0, (hipStream_t)stream, a, (u32x4*)sink);
  else
    hipLaunchKernelGGL(paged_read_probe_kernel<64>, dim3((unsigned)count), dim3(256), 0, (hipStream_t)stream, a, (u32x4*)sink);
  VKV_HIP(hipGetLastError());
  return VKV_OK;
}

int kv_attn_check(vkv_pool* p, void* workspace, void* stream) {
  int st = check_bound(p, workspace, "kv_attn_check");
  if (st != VKV_OK) return st;
  VKV_HIP(hipStreamSynchronize((hipStream_t)stream));
  uint32_t flag = 0;
  VKV_HIP(hipMemcpy(&flag, (char*)workspace + p->ws.header, 4, hipMemcpyDeviceToHost));
  if (flag) { set_error("kv_attn_check: a slice met a block-table entry outside the pool"); return VKV_E_STATE; }
  return VKV_OK;
}

int kv_attn_run_layer(vkv_pool* p, int32_t layer, int32_t* cursor, const void* q, const int32_t* table,
                      int32_t max_blk, void* workspace, void* out, float scale, int32_t max_inflight,
                      void* stream) {
  int st = check_slice_args(p, layer, q, table, max_blk, workspace, out, "kv_attn_run_layer");
  if (st != VKV_OK) return st;
  const int32_t n_slices = (int32_t)p->slice_start.size() - 1;
  hipStream_t hs = (hipStream_t)stream;
  return run_slices(p, cursor, n_slices, max_inflight, hs, "kv_attn_run_layer",
                    [&](int32_t s, hipStream_t on) {
                      return launch_slice(p, layer, s, q, table, max_blk, workspace, out, scale, on);
                    },
                    0, nullptr);
}

int kv_sched_set_overlap(vkv_pool* p, int32_t enable) {
  if (!p) { set_error("kv_sched_set_overlap: null pool"); return VKV_E_INVAL; }
  if (p->broken) { set_error("kv_sched_set_overlap: pool unusable after a HIP failure"); return VKV_E_HIP; }
  if (enable) {
    // created here, not on first use: the memory thread reads the handle during its grace wait
    if (!p->aux_stream) VKV_HIP(hipStreamCreateWithFlags(&p->aux_stream, hipStreamNonBlocking));
    if (!p->fork_ev) VKV_HIP(hipEventCreateWithFlags(&p->fork_ev, hipEventDisableTiming));
    if (!p->join_ev) VKV_HIP(hipEventCreateWithFlags(&p->join_ev, hipEventDisableTiming));
  }
  p->overlap = enable != 0;
  return VKV_OK;
}

}  // extern "C"
