// Host side of the preemptible decode attention: work plan, workspace binding, slice launches,
// the slice scheduler with the yield test, and the reads-only probe launcher.  The kernels are
// in attn_kernel.inc.
#include "vkv_internal.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <functional>
#include <thread>

namespace vkv {

#include "attn_kernel.inc"

// ---- scratch of the entry point that allocates nothing ---------------------------------
// paged_decode_attn_layer_static keeps its progress counters and per-item partial results here
// instead of in a caller-provided workspace.  Every GPU holds its own copy of the array at its
// own address; the name below is only a host-side stand-in for it, so host code looks the
// device address up once per device and uses that pointer everywhere.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char static_scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[kMaxDevices] = {};

// Device address of static_scratch on the current device (looked up on the first call there).
int static_scratch_for_current_device(void** out) {
  int dev = -1;
  VKV_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) { set_error("device ordinal %d not supported", dev); return VKV_E_INVAL; }
  std::lock_guard<std::mutex> g(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    VKV_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(static_scratch)));
    if (!ptr) { set_error("hipGetSymbolAddress gave no address for the static scratch"); return VKV_E_HIP; }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return VKV_OK;
}

__global__ void zero_words_kernel(uint32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
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

// the kernel parameters every launch of a planned layer shares
static AttnParams layer_params(vkv_pool* p, int32_t layer, const void* q, const int32_t* table, int32_t max_blk,
                               void* workspace, void* out, float scale) {
  const int D = p->cfg.head_dim;
  char* ws = (char*)workspace;
  AttnParams a{};   // every field the launch does not set is zero (no progress report, no dense grid)
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
  a.max_blk = max_blk;
  a.Hq = p->cfg.num_q_heads;
  a.Hkv = p->cfg.num_kv_heads;
  a.G = p->G;
  a.NB = p->cfg.num_blocks;
  a.scale_log2 = (scale != 0.f ? scale : 1.0f / std::sqrt((float)D)) * 1.4426950408889634f;
  return a;
}

static int launch_slice(vkv_pool* p, int32_t layer, int32_t slice, const void* q, const int32_t* table,
                        int32_t max_blk, void* workspace, void* out, float scale, hipStream_t st, bool defer_merge) {
  const int32_t first = p->slice_start[slice], count = p->slice_start[slice + 1] - first;
  const int D = p->cfg.head_dim;
  AttnParams a = layer_params(p, layer, q, table, max_blk, workspace, out, scale);
  a.item_first = first;
  a.defer_merge = defer_merge ? 1 : 0;
  if (p->report_seq) {   // the scheduler counts this launch
    a.started = p->progress_dev;
    a.seq = p->report_seq;
  }
  ProfKernel prof(p, VKV_PROF_SLICE, slice);
  if (D == 128)
    prof.launch(paged_decode_attn_slice_kernel<128, false>, dim3((unsigned)count), dim3(256), st, a);
  else
    prof.launch(paged_decode_attn_slice_kernel<64, false>, dim3((unsigned)count), dim3(256), st, a);
  VKV_HIP(hipGetLastError());
  return VKV_OK;
}

// the merge of a layer whose slices were launched with defer_merge, behind all of them
static int launch_layer_merge(vkv_pool* p, int32_t layer, const void* q, const int32_t* table, int32_t max_blk,
                              void* workspace, void* out, float scale, hipStream_t st) {
  const AttnParams a = layer_params(p, layer, q, table, max_blk, workspace, out, scale);
  const unsigned grid = (unsigned)(p->num_seqs * p->cfg.num_kv_heads);
  if (p->cfg.head_dim == 128)
    hipLaunchKernelGGL(attn_merge_kernel<128>, dim3(grid), dim3(256), 0, st, a);
  else
    hipLaunchKernelGGL(attn_merge_kernel<64>, dim3(grid), dim3(256), 0, st, a);
  VKV_HIP(hipGetLastError());
  return VKV_OK;
}

static int check_slice_args(vkv_pool* p, int32_t layer, const void* q, const int32_t* table, int32_t max_blk,
                            void* workspace, void* out, const char* who) {
  int st = check_bound(p, workspace, who);
  if (st != VKV_OK) return st;
  if (!p->cfg.base) { set_error("%s: pool has no device memory", who); return VKV_E_INVAL; }
  if (layer < 0 || layer >= p->cfg.num_layers) { set_error("%s: layer %d out of range", who, layer); return VKV_E_INVAL; }
  if (!q || !table || !out || (uintptr_t)q % 16 || (uintptr_t)out % 16) {
    set_error("%s: q and out (16-byte aligned) and block_table must be given", who);
    return VKV_E_INVAL;
  }
  if (max_blk < p->max_ctx_blocks) {
    set_error("%s: block table has %d columns, the plan needs %d", who, max_blk, p->max_ctx_blocks);
    return VKV_E_INVAL;
  }
  return VKV_OK;
}

__global__ void progress_marker_kernel(uint32_t* word, uint32_t value) {
  __hip_atomic_store(word, value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

int ensure_progress_words(vkv_pool* p) {
  if (p->progress_host) return VKV_OK;
  void* h = nullptr;
  VKV_HIP(hipHostMalloc(&h, 256, hipHostMallocDefault));
  std::memset(h, 0, 256);
  void* d = nullptr;
  hipError_t e = hipHostGetDevicePointer(&d, h, 0);
  if (e != hipSuccess) { (void)hipHostFree(h); return hip_fail(e, "hipHostGetDevicePointer"); }
  p->progress_host = (volatile uint32_t*)h;
  p->progress_dev = (uint32_t*)d;
  return VKV_OK;
}

// waits (polling pinned host memory; no runtime call) until *word has reached `want`
static void wait_progress(const volatile uint32_t* word, uint32_t want) {
  for (int spins = 0; (int32_t)(__atomic_load_n(word, __ATOMIC_ACQUIRE) - want) < 0; ++spins) {
    if (spins < 4096) __builtin_ia32_pause();
    else std::this_thread::sleep_for(std::chrono::microseconds(2));
  }
}

// Slice scheduler shared by decode and prefill: issues steps *cursor .. n_slices + n_tail - 1
// (slices through `launch`, then n_tail follow-up steps through `tail`, all on the caller's
// stream), keeping at most max_inflight launches unfinished; that state persists across calls.
// Stops at a step boundary when the yield flag is set.
// How the lead over the GPU is bounded:
//   - event ring: an event is recorded behind every launch and the host waits for the event of the
//     launch max_inflight back.  An event record between two kernels costs several microseconds of
//     GPU time, which does not matter when launches overlap on two streams and is used there, for
//     steps whose kernels do not report progress (launches_report false), and for max_inflight 1.
//   - progress words: every launch stores its number in pinned host memory when it starts, i.e. when
//     all earlier launches of the stream have finished, and the host enqueues launch n once launch
//     n - max_inflight + 1 has started; kernels follow each other with nothing in between.  A drain
//     enqueues a one-thread marker kernel behind the last launch and polls for it.
// With overlap on, odd slices go to a second stream the pool owns (forked from and joined back
// into the caller's stream inside this call), so the workgroups of the next slice fill the
// compute units the tail of the previous one leaves idle; slices of one layer are independent
// (results are merged through per-item partials), so their order does not matter.
int run_slices(vkv_pool* p, int32_t* cursor, int32_t n_slices, int32_t max_inflight, hipStream_t hs,
               const char* who, const std::function<int(int32_t, hipStream_t)>& launch, int32_t n_tail,
               const std::function<int(int32_t)>& tail, bool launches_report,
               const std::function<int()>& after_slices) {
  if (!cursor || *cursor < 0 || *cursor > n_slices + n_tail || max_inflight < 1 || max_inflight > kMaxInflight) {
    set_error("%s: bad cursor or max_inflight", who);
    return VKV_E_INVAL;
  }
  int st = VKV_OK;
  const bool two = p->overlap && p->aux_stream && max_inflight >= 2 && n_slices - *cursor >= 2;
  const bool words = launches_report && !two && max_inflight >= 2 && n_tail == 0;
  const int mode = words ? 2 : 1;

  auto drain_ring = [&]() -> int {
    for (; p->inflight_count > 0; --p->inflight_count, p->inflight_head = (p->inflight_head + 1) % p->inflight_cap)
      VKV_HIP(hipEventSynchronize(p->inflight_ev[p->inflight_head]));
    p->inflight_head = 0;
    return VKV_OK;
  };
  auto drain_words = [&]() -> int {
    // a marker behind everything enqueued so far; it runs when the last launch has finished
    const uint32_t mark = ++p->drain_seq;
    hipLaunchKernelGGL(progress_marker_kernel, dim3(1), dim3(1), 0, hs, p->progress_dev + 1, mark);
    VKV_HIP(hipGetLastError());
    wait_progress(p->progress_host + 1, mark);
    // the slices are done; the marker itself is about to retire: the stream is idle a moment later
    for (;;) {
      const hipError_t q = hipStreamQuery(hs);
      if (q == hipSuccess) break;
      if (q != hipErrorNotReady) return hip_fail(q, "hipStreamQuery");
      __builtin_ia32_pause();
    }
    return VKV_OK;
  };
  auto drain = [&]() -> int { return p->sched_mode == 2 ? drain_words() : drain_ring(); };

  if (mode == 2 && (st = ensure_progress_words(p)) != VKV_OK) return st;
  if (mode == 1)
    for (int i = 0; i < max_inflight; ++i)
      if (!p->inflight_ev[i]) VKV_HIP(hipEventCreateWithFlags(&p->inflight_ev[i], hipEventDisableTiming));
  if (p->sched_mode != mode || (mode == 1 && p->inflight_cap != max_inflight)) {
    // another way of counting from here on: nothing of the old way may be left in flight
    if (p->sched_mode != 0 && (st = drain()) != VKV_OK) return st;
    p->sched_mode = mode;
    p->inflight_cap = max_inflight;
  }

  // one more launch may be enqueued once fewer than max_inflight are unfinished
  auto admit = [&]() -> int {
    if (mode == 2) {
      // launch n may go once launch n - max_inflight + 1 has started: then at most max_inflight - 1
      // earlier launches are unfinished (one of them running)
      const uint32_t n = p->launch_seq + 1;
      if (n > (uint32_t)(max_inflight - 1)) wait_progress(p->progress_host, n - (uint32_t)(max_inflight - 1));
      return VKV_OK;
    }
    if (p->inflight_count == max_inflight) {
      VKV_HIP(hipEventSynchronize(p->inflight_ev[p->inflight_head]));
      p->inflight_head = (p->inflight_head + 1) % max_inflight;
      --p->inflight_count;
    }
    return VKV_OK;
  };
  auto track = [&](hipStream_t on) -> int {
    if (mode == 2) return VKV_OK;
    VKV_HIP(hipEventRecord(p->inflight_ev[(p->inflight_head + p->inflight_count) % max_inflight], on));
    ++p->inflight_count;
    return VKV_OK;
  };
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
  auto yielded = [&](int32_t at) -> int {
    int r = drain();
    if (r != VKV_OK) return r;
    if ((r = join()) != VKV_OK) return r;
    *cursor = at;
    return VKV_YIELDED;
  };
  for (int32_t s = *cursor; s < n_slices; ++s) {
    if (p->yield_flag.load(std::memory_order_acquire)) return yielded(s);
    const hipStream_t on = (two && (s & 1)) ? p->aux_stream : hs;
    if ((st = admit()) != VKV_OK) return st;
    // admit() may have waited for up to one slice: a request that came in meanwhile is honoured now
    if (p->yield_flag.load(std::memory_order_acquire)) return yielded(s);
    p->report_seq = mode == 2 ? ++p->launch_seq : 0;
    st = launch(s, on);
    p->report_seq = 0;
    if (st != VKV_OK) return st;
    if ((st = track(on)) != VKV_OK) return st;
    if (on != hs) aux_used = true;
    // what belongs behind the last slice goes out with it, on the caller's stream, once the second
    // stream's slices are joined: no yield test lies between the two
    if (s == n_slices - 1 && after_slices) {
      if ((st = join()) != VKV_OK) return st;
      if ((st = after_slices()) != VKV_OK) return st;
    }
  }
  if ((st = join()) != VKV_OK) return st;
  for (int32_t t = std::max(*cursor, n_slices) - n_slices; t < n_tail; ++t) {
    if (p->yield_flag.load(std::memory_order_acquire)) return yielded(n_slices + t);
    if ((st = admit()) != VKV_OK) return st;
    if (p->yield_flag.load(std::memory_order_acquire)) return yielded(n_slices + t);
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
    if (ctx[s] < 0) { set_error("kv_attn_plan: sequence %d has context length %d (< 0)", s, ctx[s]); return VKV_E_INVAL; }
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
  if (!work.empty()) starts.push_back((int32_t)work.size());   // an empty batch has no slice

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
  return launch_slice(p, layer, slice, q, table, max_blk, workspace, out, scale, (hipStream_t)stream, false);
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
  // Where a layer is many launches its split sequences are merged once, behind the last slice (issued
  // with it: a yield lands before the last slice or after the merge), not by the last arriver inside the
  // slices; the bits are the same.  A layer is resumed the way it was begun: the rule depends on the plan only.
  const bool defer = n_slices >= kDeferMergeMinSlices;
  return run_slices(p, cursor, n_slices, max_inflight, hs, "kv_attn_run_layer",
                    [&](int32_t s, hipStream_t on) {
                      return launch_slice(p, layer, s, q, table, max_blk, workspace, out, scale, on, defer);
                    },
                    0, nullptr, true,
                    defer ? std::function<int()>([&]() {
                      return launch_layer_merge(p, layer, q, table, max_blk, workspace, out, scale, hs);
                    }) : std::function<int()>());
}

int paged_decode_attn_layer_static(vkv_pool* p, int32_t layer, const void* q, const int32_t* table, int32_t max_blk,
                                   const int32_t* ctx_len_dev, int32_t num_seqs, int32_t max_ctx_tokens,
                                   int32_t chunk_tokens, void* out, uint32_t* err_flag_dev, float scale, void* stream) {
  const char* who = "paged_decode_attn_layer_static";
  if (!p) { set_error("%s: null pool", who); return VKV_E_INVAL; }
  if (p->broken) { set_error("%s: pool unusable after a HIP failure", who); return VKV_E_HIP; }
  if (!p->cfg.base) { set_error("%s: pool has no device memory", who); return VKV_E_INVAL; }
  if (layer < 0 || layer >= p->cfg.num_layers) { set_error("%s: layer %d out of range", who, layer); return VKV_E_INVAL; }
  if (!q || !table || !ctx_len_dev || !out || (uintptr_t)q % 16 || (uintptr_t)out % 16 || (uintptr_t)err_flag_dev % 4) {
    set_error("%s: q and out (16-byte aligned), block_table and ctx_len must be given", who);
    return VKV_E_INVAL;
  }
  if (chunk_tokens < kGroupTokens || chunk_tokens % kGroupTokens || chunk_tokens > kMaxChunkTokens) {
    set_error("%s: chunk_tokens must be a multiple of %d in [%d, %d]", who, kGroupTokens, kGroupTokens, kMaxChunkTokens);
    return VKV_E_INVAL;
  }
  const int B = p->cfg.block_tokens, Hkv = p->cfg.num_kv_heads, D = p->cfg.head_dim, G = p->G;
  if (num_seqs < 1 || max_ctx_tokens < 1 || max_blk < 1 || (int64_t)max_ctx_tokens > (int64_t)max_blk * B) {
    set_error("%s: need num_seqs >= 1 and 1 <= max_ctx_tokens <= max_blk * %d", who, B);
    return VKV_E_INVAL;
  }
  const int64_t max_chunks = ((int64_t)max_ctx_tokens + chunk_tokens - 1) / chunk_tokens;
  if (max_chunks * G * 8 > kMergeLdsBytes) {
    set_error("%s: %lld chunks per sequence is too many for group size %d; raise chunk_tokens", who,
              (long long)max_chunks, G);
    return VKV_E_INVAL;
  }
  const int64_t n_items = (int64_t)num_seqs * max_chunks * Hkv;
  // scratch: [0,256) header (word 0 = flag when the caller gives none) | done | (max, sum) | weighted V sums
  const uint64_t off_done = 256;
  const uint64_t off_ml = align_up(off_done + (uint64_t)num_seqs * Hkv * 4, 256);
  const uint64_t off_acc = align_up(off_ml + (uint64_t)n_items * G * 2 * 4, 256);
  const uint64_t need = max_chunks > 1 ? off_acc + (uint64_t)n_items * G * D * 4 : off_ml;
  if (n_items > 0x7FFFFFF0ll || need > kStaticScratchBytes) {
    set_error("%s: %d sequences x %lld chunks x %d kv heads need %llu bytes of scratch, the static buffer holds %llu; "
              "raise chunk_tokens, split the batch, or use paged_decode_attn_slice with a workspace",
              who, num_seqs, (long long)max_chunks, Hkv, (unsigned long long)need,
              (unsigned long long)kStaticScratchBytes);
    return VKV_E_NOSPACE;
  }
  void* base_v = nullptr;
  int st = static_scratch_for_current_device(&base_v);
  if (st != VKV_OK) return st;
  char* sc = (char*)base_v;
  hipStream_t hs = (hipStream_t)stream;
  // the counters (and the flag word) must start at zero whatever an earlier call left behind; a fill
  // kernel, not a memset, so that the call can be recorded into a graph
  const int n_zero = (int)((off_ml - 0) / 4);
  hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)((n_zero + 255) / 256)), dim3(256), 0, hs, (uint32_t*)sc, n_zero);
  VKV_HIP(hipGetLastError());
  AttnParams a{};
  a.pool = (const uint16_t*)p->cfg.base + (uint64_t)layer * ((uint64_t)2 * Hkv * 16 * D);
  a.q = (const uint16_t*)q;
  a.table = table;
  a.part_acc = (float*)(sc + off_acc);
  a.part_ml = (float*)(sc + off_ml);
  a.done = (int32_t*)(sc + off_done);
  a.out = (float*)out;
  a.err = err_flag_dev ? err_flag_dev : (uint32_t*)sc;
  a.block_elems = p->block_elems;
  a.v_off = (uint32_t)(Hkv * 16 * D);
  a.max_blk = max_blk;
  a.Hq = p->cfg.num_q_heads;
  a.Hkv = Hkv;
  a.G = G;
  a.NB = p->cfg.num_blocks;
  a.chunk_blocks = chunk_tokens / B;
  a.scale_log2 = (scale != 0.f ? scale : 1.0f / std::sqrt((float)D)) * 1.4426950408889634f;
  a.ctx_len = ctx_len_dev;
  a.max_chunks = (int32_t)max_chunks;
  a.max_ctx = max_ctx_tokens;
  ProfKernel prof(p, VKV_PROF_SLICE, 0);
  if (D == 128)
    prof.launch(paged_decode_attn_slice_kernel<128, true>, dim3((unsigned)n_items), dim3(256), hs, a);
  else
    prof.launch(paged_decode_attn_slice_kernel<64, true>, dim3((unsigned)n_items), dim3(256), hs, a);
  VKV_HIP(hipGetLastError());
  return VKV_OK;
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
