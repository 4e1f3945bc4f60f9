// Native driver for hardware-counter runs: the Llama-3-8B-shaped decode + reclamation step
// through the C ABI, with no Python in the process (rocprofv3 --pmc -- ./vkv_pmc_driver).
// It is also the smallest complete example of the call sequence a framework would use.
//
//   vkv_pmc_driver [layers=32] [steps=2] [pool_GiB=40] [prefill_tokens=0] [prefill_slice_MiB=1024] [prefill_chunk=4096]
//   vkv_pmc_driver state=<file> [layers to run=all] [steps=2]
//
// The second form runs a workload written by `python -m synth.dump_state <workload> <seed> <file>`:
// the benchmark's own contexts, block tables, slice and chunk sizes.  Both forms end with three reads
// and three fills of exactly 1 GiB, which give the byte counters their scale.
//
// With prefill_tokens > 0 one layer of causal prefill of the newest min(context, prefill_tokens)
// tokens of every sequence runs after the decode/reclaim steps.
//
// Inputs are synthetic: contexts ~ lognormal(median 2048, sigma 0.7) clipped to [16, 8192],
// 64 sequences, 32 query / 8 KV heads of 128, 70 % of the pool's 2 MiB blocks live at random
// positions, the top 10 % of the pool reclaimed.  Values are a cheap integer hash turned into
// small bf16 numbers; counters do not depend on them.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <numeric>
#include <random>
#include <vector>

#include "valvekv.h"

#define CK(x)                                                                        \
  do {                                                                               \
    hipError_t e_ = (x);                                                             \
    if (e_ != hipSuccess) {                                                          \
      std::fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));            \
      std::exit(1);                                                                  \
    }                                                                                \
  } while (0)
#define VK(x)                                                                        \
  do {                                                                               \
    int s_ = (x);                                                                    \
    if (s_ < 0) {                                                                    \
      std::fprintf(stderr, "%s failed (%d): %s\n", #x, s_, vkv_last_error());        \
      std::exit(1);                                                                  \
    }                                                                                \
  } while (0)

// bf16 values in (-2, 2) from a hash of the element index
__global__ void fill_bf16(uint16_t* p, size_t n, uint32_t seed) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    uint32_t h = (uint32_t)i * 2654435761u ^ (uint32_t)(i >> 32) ^ seed;
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
    p[i] = (uint16_t)(((h & 0x8000u)) | 0x3F00u | (h & 0xFFu));   // sign, exponent of 0.5..2, 8 mantissa bits (7 used)
  }
}

// A workload written by `python -m synth.dump_state <workload> <seed> <file>`: the benchmark's own
// geometry, context lengths, block tables and live blocks.
struct State {
  int L = 0, Hq = 0, Hkv = 0, D = 0, NB = 0, bph = 0, S = 0, n_rows = 0, max_blk = 0, lo = 0, hi = 0, chunk_tokens = 0;
  uint64_t slice_bytes = 0, reclaim_chunk_bytes = 0;
  std::vector<int32_t> ctx, tables, live_ids;
};

static bool read_state(const char* path, State& st) {
  FILE* f = std::fopen(path, "rb");
  if (!f) return false;
  int32_t h[16];
  int64_t w[2];
  bool ok = std::fread(h, 4, 16, f) == 16 && std::fread(w, 8, 2, f) == 2 && h[0] == 0x53564B56 && h[1] == 1;
  if (ok) {
    st.L = h[2]; st.Hq = h[3]; st.Hkv = h[4]; st.D = h[5]; st.NB = h[6]; st.bph = h[7]; st.S = h[8];
    st.n_rows = h[9]; st.max_blk = h[10]; st.lo = h[11]; st.hi = h[12]; st.chunk_tokens = h[13];
    st.slice_bytes = (uint64_t)w[0];
    st.reclaim_chunk_bytes = (uint64_t)w[1];
    ok = st.L > 0 && st.S > 0 && st.NB > 0 && st.n_rows >= st.S && st.max_blk > 0;
  }
  if (ok) {
    st.ctx.resize((size_t)st.S);
    st.tables.resize((size_t)st.n_rows * st.max_blk);
    std::vector<uint8_t> live((size_t)st.NB);
    ok = std::fread(st.ctx.data(), 4, st.ctx.size(), f) == st.ctx.size() &&
         std::fread(st.tables.data(), 4, st.tables.size(), f) == st.tables.size() &&
         std::fread(live.data(), 1, live.size(), f) == live.size();
    for (int b = 0; ok && b < st.NB; ++b)
      if (live[(size_t)b]) st.live_ids.push_back(b);
  }
  std::fclose(f);
  return ok;
}

int main(int argc, char** argv) {
  const bool from_file = argc > 1 && std::strncmp(argv[1], "state=", 6) == 0;
  State sf;
  if (from_file && !read_state(argv[1] + 6, sf)) { std::fprintf(stderr, "cannot read state file %s\n", argv[1] + 6); return 1; }
  // state=<file> [layers to run = all] [steps = 2]   |   [layers=32] [steps=2] [pool_GiB=40] [prefill ...]
  const int L = from_file ? sf.L : (argc > 1 ? std::atoi(argv[1]) : 32);
  const int L_run = from_file && argc > 2 ? std::min(L, std::max(1, std::atoi(argv[2]))) : L;
  const int steps = from_file ? (argc > 3 ? std::atoi(argv[3]) : 2) : (argc > 2 ? std::atoi(argv[2]) : 2);
  const int pool_gib = !from_file && argc > 3 ? std::atoi(argv[3]) : 40;
  const int prefill_tokens = !from_file && argc > 4 ? std::atoi(argv[4]) : 0;
  const uint64_t prefill_slice = (uint64_t)(!from_file && argc > 5 ? std::atoi(argv[5]) : 1024) << 20;
  const int prefill_chunk = !from_file && argc > 6 ? std::atoi(argv[6]) : 4096;
  const int S = from_file ? sf.S : 64, Hq = from_file ? sf.Hq : 32, Hkv = from_file ? sf.Hkv : 8,
            D = from_file ? sf.D : 128, B = 16;
  const size_t block_elems = (size_t)L * 2 * Hkv * B * D;
  const size_t block_bytes = block_elems * 2;
  const int bph = from_file ? sf.bph : 32;
  const int NB = from_file ? sf.NB : (int)(((size_t)pool_gib << 30) / block_bytes / bph * bph);
  const int max_blk = from_file ? sf.max_blk : 8192 / B;
  const uint64_t slice_bytes = from_file ? sf.slice_bytes : 1ull << 30;
  const int chunk_tokens = from_file ? sf.chunk_tokens : 1024;
  const uint64_t reclaim_chunk = from_file ? sf.reclaim_chunk_bytes : 0;

  std::vector<int32_t> ctx, tables, live_ids;
  if (from_file) {
    ctx = sf.ctx;
    tables = sf.tables;
    live_ids = sf.live_ids;
  } else {
    std::mt19937_64 rng(0);
    std::lognormal_distribution<double> ln(std::log(2048.0), 0.7);
    ctx.resize(S);
    for (auto& c : ctx) c = (int32_t)std::min(8192.0, std::max(16.0, std::nearbyint(ln(rng))));
    std::vector<int32_t> ids(NB);
    std::iota(ids.begin(), ids.end(), 0);
    std::shuffle(ids.begin(), ids.end(), rng);
    const int n_live = (int)(0.7 * NB);
    tables.assign((size_t)S * max_blk, -1);
    size_t cur = 0;
    for (int s = 0; s < S; ++s)
      for (int j = 0; j < (ctx[s] + B - 1) / B; ++j) tables[(size_t)s * max_blk + j] = ids[cur++];
    if ((int)cur > n_live) { std::fprintf(stderr, "batch does not fit\n"); return 1; }
    // background blocks get table rows of their own
    const size_t bg = n_live - cur, bg_rows = (bg + max_blk - 1) / max_blk;
    tables.resize((size_t)(S + bg_rows) * max_blk, -1);
    for (size_t i = 0; i < bg; ++i) tables[(size_t)S * max_blk + i] = ids[cur + i];
    live_ids.assign(ids.begin(), ids.begin() + n_live);
  }
  const int n_live = (int)live_ids.size();

  uint16_t *pool_d, *q_d;
  int32_t *tables_d, *tables0_d, *remap_d;
  float* out_d;
  CK(hipMalloc(&pool_d, (size_t)NB * block_bytes));
  CK(hipMalloc(&q_d, (size_t)L * S * Hq * D * 2));
  CK(hipMalloc(&tables_d, tables.size() * 4));
  CK(hipMalloc(&tables0_d, tables.size() * 4));
  CK(hipMalloc(&remap_d, (size_t)NB * 4));
  CK(hipMalloc(&out_d, (size_t)S * Hq * D * 4));
  hipLaunchKernelGGL(fill_bf16, dim3(8192), dim3(256), 0, 0, pool_d, (size_t)NB * block_elems, 1u);
  hipLaunchKernelGGL(fill_bf16, dim3(256), dim3(256), 0, 0, q_d, (size_t)L * S * Hq * D, 2u);
  CK(hipMemcpy(tables0_d, tables.data(), tables.size() * 4, hipMemcpyHostToDevice));
  CK(hipMemcpy(tables_d, tables0_d, tables.size() * 4, hipMemcpyDeviceToDevice));
  CK(hipDeviceSynchronize());

  vkv_pool_config cfg{};
  cfg.num_layers = L; cfg.num_q_heads = Hq; cfg.num_kv_heads = Hkv; cfg.head_dim = D; cfg.block_tokens = B;
  cfg.num_blocks = NB; cfg.blocks_per_handle = bph; cfg.base = pool_d; cfg.bytes = (uint64_t)NB * block_bytes;
  vkv_pool* pool = nullptr;
  VK(kv_pool_init(&cfg, &pool));
  VK(kv_pool_adopt(pool, live_ids.data(), n_live));

  vkv_attn_plan_info info{};
  VK(kv_attn_plan(pool, ctx.data(), S, slice_bytes, chunk_tokens, &info));
  void* ws;
  CK(hipMalloc(&ws, info.workspace_bytes));
  VK(kv_attn_bind(pool, ws, info.workspace_bytes, nullptr));
  const int lo = from_file ? sf.lo : (NB - NB / 10) / bph * bph, hi = from_file ? sf.hi : NB;
  vkv_reclaim_stats rs{};
  std::vector<int32_t> remap_h(NB);
  VK(kv_reclaim_plan(pool, lo, hi, remap_h.data(), &rs));
  std::vector<int32_t> src, dst;
  for (int b = lo; b < hi; ++b)
    if (remap_h[b] != b) { src.push_back(b); dst.push_back(remap_h[b]); }

  std::printf("L=%d S=%d pool=%d blocks of %zu KiB; items %d slices %d; kv bytes/layer %llu; "
              "reclaim [%d,%d): %d blocks = %llu bytes moved\n",
              L, S, NB, block_bytes >> 10, info.n_items, info.n_slices,
              (unsigned long long)info.kv_bytes_per_layer, lo, hi, rs.blocks_moved, (unsigned long long)rs.bytes_moved);
  for (int step = 0; step < steps; ++step) {
    for (int layer = 0; layer < L_run; ++layer) {
      int32_t cursor = 0;
      VK(kv_attn_run_layer(pool, layer, &cursor, q_d + (size_t)layer * S * Hq * D, tables_d, max_blk, ws, out_d, 0.f, 2,
                           nullptr));
    }
    VK(kv_reclaim_range(pool, lo, hi, tables_d, (int64_t)tables.size(), reclaim_chunk, 0, nullptr, nullptr, remap_d, 0, &rs));
    // the online tenant returns the range; rewind the bookkeeping (the sources were left intact)
    VK(kv_pool_return_range(pool, lo, hi));
    VK(kv_pool_free(pool, dst.data(), (int32_t)dst.size()));
    VK(kv_pool_adopt(pool, src.data(), (int32_t)src.size()));
    CK(hipMemcpy(tables_d, tables0_d, tables.size() * 4, hipMemcpyDeviceToDevice));
  }
  VK(kv_attn_check(pool, ws, nullptr));
  CK(hipDeviceSynchronize());
  {
    // Launches of known size, for scaling the byte counters: a read of exactly 1 GiB (probe_read_kernel,
    // stores nothing) and a fill of exactly 1 GiB (fill_bf16, loads nothing), three of each.
    const size_t cal = 1ull << 30;
    uint16_t* cal_d;
    void* sink_d;
    CK(hipMalloc(&cal_d, cal));
    CK(hipMalloc(&sink_d, 256));
    for (int i = 0; i < 3; ++i) {
      hipLaunchKernelGGL(fill_bf16, dim3(8192), dim3(256), 0, 0, cal_d, cal / 2, 7u + i);
      VK(kv_probe_read(cal_d, cal, sink_d, nullptr));
    }
    CK(hipDeviceSynchronize());
    CK(hipFree(cal_d));
    CK(hipFree(sink_d));
  }
  if (prefill_tokens > 0) {
    std::vector<int32_t> q_len(S);
    for (int s = 0; s < S; ++s) q_len[s] = std::min(ctx[s], prefill_tokens);
    vkv_prefill_plan_info pinfo{};
    VK(kv_prefill_plan(pool, ctx.data(), q_len.data(), S, prefill_slice, prefill_chunk, &pinfo));
    void* pws;
    uint16_t* pq;
    float* pout;
    CK(hipMalloc(&pws, pinfo.workspace_bytes));
    CK(hipMalloc(&pq, (size_t)pinfo.total_q * Hq * D * 2));
    CK(hipMalloc(&pout, (size_t)pinfo.total_q * Hq * D * 4));
    hipLaunchKernelGGL(fill_bf16, dim3(1024), dim3(256), 0, 0, pq, (size_t)pinfo.total_q * Hq * D, 3u);
    VK(kv_prefill_bind(pool, pws, pinfo.workspace_bytes, nullptr));
    int32_t cursor = 0;
    VK(kv_prefill_run_layer(pool, 0, &cursor, pq, tables_d, max_blk, pws, pout, 0.f, 2, nullptr));
    VK(kv_prefill_check(pool, pws, nullptr));
    std::printf("prefill: %d rows, %d items, %d slices, %.3e flops, %llu kv bytes\n", pinfo.total_q, pinfo.n_items,
                pinfo.n_slices, pinfo.flops_per_layer, (unsigned long long)pinfo.kv_bytes_per_layer);
  }
  VK(kv_pool_destroy(pool));
  std::printf("done\n");
  return 0;
}
