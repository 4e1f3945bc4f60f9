// KV reclamation: empty a block range by relocating its live blocks and rewriting block
// tables (the problem of paper Section 5, "Sub-layer memory reclamation": hand handles
// to the online tenant promptly, with no access to handed-over memory afterwards and
// without killing the offline job).  The copy is HBM-bound: every live byte of the
// range is read once and written once.
#include "vkv_internal.h"

#include <algorithm>
#include <chrono>
#include <thread>

namespace vkv {

// ---- kernels ----------------------------------------------------------------------

constexpr int kCopyThreads = 256;
// 16-byte vectors in flight per thread: 16 (64 KiB per workgroup) or, for blocks of at least 1 MiB
// that divide evenly, 32 (128 KiB per workgroup; 3-4 % faster there, slower on smaller blocks)
constexpr int kCopyUnrollSmall = 16, kCopyUnrollLarge = 32;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// One workgroup copies one piece (64 or 128 KiB) of one live block of [first_src, first_src + gridDim.x)
// to remap[src].  Each wave owns a contiguous quarter of the piece and moves it with 16 or 32 loads in
// flight, then as many stores, all non-temporal (the data is not read again soon): requests of one wave
// that follow each other in address measured 15 % more copy bandwidth than rows interleaved over the
// four waves (6.1 against 5.3 TB/s of traffic).  Blocks with remap[src] == src (free, nothing to move)
// exit at once.
template <int kCopyUnroll>
__global__ __launch_bounds__(kCopyThreads) void kv_block_relocate_kernel(
    u32x4* __restrict__ pool, const int32_t* __restrict__ remap, int32_t first_src,
    uint32_t block_vecs /* 16-byte vectors per block */) {
  const int32_t src = first_src + (int32_t)blockIdx.x;
  const int32_t dst = remap[src];
  if (dst == src) return;
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint32_t v0 = blockIdx.y * (uint32_t)(kCopyThreads * kCopyUnroll) + wave * (kCopyUnroll * 64u) + lane;
  const u32x4* __restrict__ s = pool + (size_t)src * block_vecs;
  u32x4* __restrict__ d = pool + (size_t)dst * block_vecs;
  u32x4 r[kCopyUnroll];
#pragma unroll
  for (int u = 0; u < kCopyUnroll; ++u) {
    const uint32_t i = v0 + u * 64u;
    if (i < block_vecs) r[u] = __builtin_nontemporal_load(s + i);
  }
#pragma unroll
  for (int u = 0; u < kCopyUnroll; ++u) {
    const uint32_t i = v0 + u * 64u;
    if (i < block_vecs) __builtin_nontemporal_store(r[u], d + i);
  }
}

__global__ __launch_bounds__(256) void block_table_rewrite_kernel(
    int32_t* __restrict__ tables, int64_t n, const int32_t* __restrict__ remap, int32_t nb) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    int32_t e = tables[i];
    if (e >= 0 && e < nb) {
      int32_t r = remap[e];
      if (r != e) tables[i] = r;
    }
  }
}

// ---- host -------------------------------------------------------------------------

static int check_range(const vkv_pool* p, int32_t lo, int32_t hi) {
  const int32_t nb = p->cfg.num_blocks, bph = p->cfg.blocks_per_handle;
  if (lo < 0 || hi > nb || lo >= hi || lo % bph || hi % bph) {
    set_error("range [%d,%d) must be non-empty, inside [0,%d) and a multiple of %d blocks", lo, hi, nb, bph);
    return VKV_E_INVAL;
  }
  for (const auto& r : p->released)
    if (lo < r.second && r.first < hi) {
      set_error("range [%d,%d) overlaps handed-over range [%d,%d)", lo, hi, r.first, r.second);
      return VKV_E_BUSY;
    }
  return VKV_OK;
}

int plan_relocation(const vkv_pool* p, int32_t lo, int32_t hi, std::vector<int32_t>& src,
                    std::vector<int32_t>& dst) {
  int st = check_range(p, lo, hi);
  if (st != VKV_OK) return st;
  src.clear();
  dst.clear();
  for (int32_t b = lo; b < hi; ++b)
    if (p->live[b]) src.push_back(b);
  const int32_t nb = p->cfg.num_blocks;
  for (int32_t b = 0; b < nb && dst.size() < src.size(); ++b) {
    if (b == lo) { b = hi - 1; continue; }
    if (p->live[b]) continue;
    if (!p->released.empty() && in_released(p, b)) continue;
    dst.push_back(b);
  }
  if (dst.size() < src.size()) {
    set_error("range [%d,%d) holds %zu live blocks, only %zu free blocks outside it", lo, hi, src.size(),
              dst.size());
    return VKV_E_NOSPACE;
  }
  return VKV_OK;
}

int launch_rewrite(vkv_pool* p, int32_t* tables, int64_t n, const int32_t* remap, int32_t nb, hipStream_t st) {
  if (n == 0) return VKV_OK;
  static vkv_pool none;   // timing records need a pool; a launch without one records nothing
  ProfScope prof(p ? p : &none, VKV_PROF_REWRITE, 0, st);
  int64_t blocks = std::min<int64_t>((n + 255) / 256, 2048);
  hipLaunchKernelGGL(block_table_rewrite_kernel, dim3((unsigned)blocks), dim3(256), 0, st, tables, n, remap, nb);
  VKV_HIP(hipGetLastError());
  return VKV_OK;
}

int grace_wait(vkv_pool* p, hipStream_t cs, hipStream_t ds) {
  if (ds != cs) {
    // slices enqueued before the rewrite finished may hold old entries (NULL is the default stream)
    VKV_HIP(hipEventRecord(p->grace_ev, ds));
    VKV_HIP(hipEventSynchronize(p->grace_ev));
  }
  if (p->aux_stream && p->aux_stream != cs) {
    // slices the scheduler sent to the pool's second stream are in the same position
    VKV_HIP(hipEventRecord(p->grace_ev, p->aux_stream));
    VKV_HIP(hipEventSynchronize(p->grace_ev));
  }
  return VKV_OK;
}

}  // namespace vkv

using namespace vkv;
using clk = std::chrono::steady_clock;

extern "C" {

int kv_reclaim_plan(vkv_pool* p, int32_t lo, int32_t hi, int32_t* remap_out, vkv_reclaim_stats* stats) {
  if (!p) { set_error("kv_reclaim_plan: null pool"); return VKV_E_INVAL; }
  std::vector<int32_t> src, dst;
  int st = plan_relocation(p, lo, hi, src, dst);
  if (st != VKV_OK) return st;
  if (remap_out) {
    for (int32_t b = 0; b < p->cfg.num_blocks; ++b) remap_out[b] = b;
    for (size_t i = 0; i < src.size(); ++i) remap_out[src[i]] = dst[i];
  }
  if (stats) {
    *stats = vkv_reclaim_stats{};
    stats->blocks_moved = (int32_t)src.size();
    stats->bytes_moved = (uint64_t)src.size() * p->block_bytes;
    stats->blocks_in_range = hi - lo;
  }
  return VKV_OK;
}

int kv_reclaim_range(vkv_pool* p, int32_t lo, int32_t hi, int32_t* tables, int64_t n_entries,
                     uint64_t chunk_bytes, uint64_t rate_cap, void* copy_stream_v, void* decode_stream_v,
                     int32_t* remap_dev, uint32_t flags, vkv_reclaim_stats* stats) {
  const auto t_begin = clk::now();
  if (!p) { set_error("kv_reclaim_range: null pool"); return VKV_E_INVAL; }
  if (p->broken) { set_error("kv_reclaim_range: pool unusable after a HIP failure"); return VKV_E_HIP; }
  if (!p->cfg.base || !remap_dev || n_entries < 0 || (n_entries > 0 && !tables)) {
    set_error("kv_reclaim_range: pool memory, remap scratch and tables must be given");
    return VKV_E_INVAL;
  }
  if (p->block_bytes % 16 || p->block_bytes / 16 > 0xFFFFFFFFull) {
    set_error("kv_reclaim_range: unsupported block size");
    return VKV_E_INVAL;
  }
  std::vector<int32_t> src, dst;
  int st = plan_relocation(p, lo, hi, src, dst);
  if (st != VKV_OK) return st;

  hipStream_t cs = (hipStream_t)copy_stream_v;
  hipStream_t ds = (hipStream_t)decode_stream_v;
  const int32_t nb = p->cfg.num_blocks;
  st = ensure_remap_stage(p);
  if (st != VKV_OK) return st;

  // From here on a failure leaves device state undefined: mark the pool broken.
  auto fail = [&](int code) { p->broken = true; return code; };

  for (int32_t b = 0; b < nb; ++b) p->remap_stage[b] = b;
  for (size_t i = 0; i < src.size(); ++i) p->remap_stage[src[i]] = dst[i];
  hipError_t he = hipMemcpyAsync(remap_dev, p->remap_stage, (size_t)nb * 4, hipMemcpyHostToDevice, cs);
  if (he != hipSuccess) return fail(hip_fail(he, "remap upload"));
  he = hipEventRecord(p->remap_ev, cs);
  if (he != hipSuccess) return fail(hip_fail(he, "hipEventRecord"));
  p->remap_inflight = true;

  // Copy launches: consecutive source ranges holding at most chunk_bytes of live data.
  const uint32_t block_vecs = (uint32_t)(p->block_bytes / 16);
  const bool large = p->block_bytes >= (1u << 20) && block_vecs % (kCopyThreads * kCopyUnrollLarge) == 0;
  const uint32_t piece_vecs = kCopyThreads * (large ? kCopyUnrollLarge : kCopyUnrollSmall);
  const uint32_t pieces = (block_vecs + piece_vecs - 1) / piece_vecs;
  const size_t per_chunk = chunk_bytes ? std::max<uint64_t>(1, chunk_bytes / p->block_bytes) : src.size();
  int32_t n_chunks = 0;
  uint64_t sent = 0;
  const int32_t planned_chunks = per_chunk ? (int32_t)((src.size() + per_chunk - 1) / per_chunk) : 0;
  {
  // one timing record brackets all copy launches of this call (index = number of launches)
  ProfScope prof(p, VKV_PROF_RELOCATE, planned_chunks, cs);
  for (size_t i = 0; i < src.size(); i += per_chunk) {
    const size_t j = std::min(src.size(), i + per_chunk);
    if (rate_cap) {
      // token bucket: this launch may start once the bytes sent so far fit under the cap
      const auto due = t_begin + std::chrono::nanoseconds((int64_t)((double)sent / (double)rate_cap * 1e9));
      std::this_thread::sleep_until(due);
    }
    const int32_t first = src[i], last = src[j - 1];
    if (large)
      hipLaunchKernelGGL(kv_block_relocate_kernel<kCopyUnrollLarge>, dim3((unsigned)(last - first + 1), pieces),
                         dim3(kCopyThreads), 0, cs, (u32x4*)p->cfg.base, (const int32_t*)remap_dev, first, block_vecs);
    else
      hipLaunchKernelGGL(kv_block_relocate_kernel<kCopyUnrollSmall>, dim3((unsigned)(last - first + 1), pieces),
                         dim3(kCopyThreads), 0, cs, (u32x4*)p->cfg.base, (const int32_t*)remap_dev, first, block_vecs);
    he = hipGetLastError();
    if (he != hipSuccess) return fail(hip_fail(he, "kv_block_relocate launch"));
    sent += (uint64_t)(j - i) * p->block_bytes;
    ++n_chunks;
  }
  }
  if (launch_rewrite(p, tables, n_entries, remap_dev, nb, cs) != VKV_OK) return fail(VKV_E_HIP);

  if (!(flags & VKV_RECLAIM_ASYNC)) {
    he = hipStreamSynchronize(cs);
    if (he != hipSuccess) return fail(hip_fail(he, "hipStreamSynchronize"));
    p->remap_inflight = false;
    if (!(flags & VKV_RECLAIM_NO_GRACE) && grace_wait(p, cs, ds) != VKV_OK) return fail(VKV_E_HIP);
  }

  for (size_t i = 0; i < src.size(); ++i) {
    p->live[src[i]] = 0;
    p->live[dst[i]] = 1;
  }
  p->hand_over(lo, hi, true);
  if (stats) {
    *stats = vkv_reclaim_stats{};
    stats->blocks_moved = (int32_t)src.size();
    stats->bytes_moved = (uint64_t)src.size() * p->block_bytes;
    stats->blocks_in_range = hi - lo;
    stats->n_chunks = n_chunks;
    stats->host_seconds = std::chrono::duration<double>(clk::now() - t_begin).count();
  }
  return VKV_OK;
}

int block_table_rewrite(int32_t* tables, int64_t n_entries, const int32_t* remap_dev, int32_t num_blocks,
                        void* stream) {
  if (n_entries < 0 || (n_entries > 0 && (!tables || !remap_dev)) || num_blocks < 1) {
    set_error("block_table_rewrite: bad argument");
    return VKV_E_INVAL;
  }
  return launch_rewrite(nullptr, tables, n_entries, remap_dev, num_blocks, (hipStream_t)stream);
}

}  // extern "C"
