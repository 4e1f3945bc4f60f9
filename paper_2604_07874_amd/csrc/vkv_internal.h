// Internal declarations shared by the translation units of libvalvekv.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>

#include <atomic>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <functional>
#include <mutex>
#include <string>
#include <utility>
#include <vector>

#include "valvekv.h"

namespace vkv {

void set_error(const char* fmt, ...);
int  hip_fail(hipError_t e, const char* what);

#define VKV_HIP(call)                                         \
  do {                                                        \
    hipError_t e_ = (call);                                   \
    if (e_ != hipSuccess) return vkv::hip_fail(e_, #call);    \
  } while (0)

constexpr int kMaxInflight = 8;
constexpr int kGroupTokens = 32;   // tokens one wave handles per loop iteration (two blocks)
constexpr int kMergeLdsBytes = 16 * 1024;   // LDS the last chunk may use for per-chunk (max, sum)
// a layer of at least this many slices merges its split sequences in one launch of its own after the last
// slice (kv_attn_run_layer) instead of inside the slices
constexpr int kDeferMergeMinSlices = 4;
constexpr int kMaxChunkTokens = 2048;   // an item's block ids fit two registers per lane

struct WorkItem {   // matches int4 on the device
  int32_t seq, kv_head, first_block, n_tokens;
};

// Byte offsets of the pieces of the attention workspace.
struct WorkspaceLayout {
  uint64_t header = 0;       // 256 bytes; word 0 = bad-table-entry flag
  uint64_t work = 0;         // WorkItem[n_items], in launch order (a permutation inside each slice)
  uint64_t seq_base = 0;     // int32[num_seqs + 1]: first item of each sequence
  uint64_t done = 0;         // int32[num_seqs][kv_heads]: chunks finished in the current layer
  uint64_t part_ml = 0;      // float[n_items][G][2]: running max (log2 units), sum of exponentials
  uint64_t part_acc = 0;     // float[n_items][G][D]: exp-weighted sum of V rows
  uint64_t total = 0;
  uint64_t upload_bytes = 0; // header + work + seq_base + done are written by kv_attn_bind
};

inline uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

inline WorkspaceLayout workspace_layout(int64_t n_items, int64_t num_seqs, int Hkv, int G, int D) {
  WorkspaceLayout w;
  w.header = 0;
  w.work = 256;
  w.seq_base = w.work + (uint64_t)n_items * sizeof(WorkItem);
  w.done = w.seq_base + (uint64_t)(num_seqs + 1) * 4;
  w.upload_bytes = w.done + (uint64_t)num_seqs * Hkv * 4;
  w.part_ml = align_up(w.upload_bytes, 256);
  w.part_acc = align_up(w.part_ml + (uint64_t)n_items * G * 2 * 4, 256);
  w.total = align_up(w.part_acc + (uint64_t)n_items * G * D * 4, 256);
  return w;
}

}  // namespace vkv

struct vkv_arena;

struct vkv_pool {
  vkv_pool_config cfg{};
  const vkv_arena* arena = nullptr;   // handle-backed memory under the pool, if the caller attached one
  int G = 1;
  uint64_t block_elems = 0;   // bf16 elements per block
  uint64_t block_bytes = 0;

  // occupancy
  std::vector<uint8_t> live;
  // handed-over ranges [first, second).  `clean` = every device block table the library was shown has
  // been rewritten and every slice that could hold an old entry has finished: only then may the
  // range's memory be unmapped.
  struct Range {
    int32_t first, second;
    bool clean;
    Range(int32_t a, int32_t b, bool c = true) : first(a), second(b), clean(c) {}
  };
  std::vector<Range> released;
  std::vector<uint8_t> handed;   // per block: 1 inside a handed-over range (kept in step with `released`)
  int64_t n_live = 0;
  void hand_over(int32_t lo, int32_t hi, bool clean) {
    released.emplace_back(lo, hi, clean);
    std::fill(handed.begin() + lo, handed.begin() + hi, (uint8_t)1);
  }

  // attention plan (host)
  bool has_plan = false;
  uint64_t plan_gen = 0;
  int32_t num_seqs = 0;
  int32_t chunk_tokens = 0;
  int32_t max_ctx_blocks = 0;                  // widest sequence in blocks
  std::vector<vkv::WorkItem> work;
  std::vector<int32_t> slice_start;
  std::vector<int32_t> seq_base;
  std::vector<int32_t> order;            // launch order of the items (a permutation inside each slice)
  vkv::WorkspaceLayout ws{};

  // binding of the plan to a device workspace
  void* bound_ws = nullptr;
  uint64_t bound_gen = 0;

  // prefill plan (host) and its binding; see prefill.hip
  struct PrefillPlan {
    bool has_plan = false;
    uint64_t gen = 0, bound_gen = 0;
    void* bound_ws = nullptr;
    int32_t num_seqs = 0, total_q = 0, max_ctx_blocks = 0, gp_shift = 0, tile_positions = 0;
    std::vector<vkv::WorkItem> work;       // .seq holds the tile id
    std::vector<int32_t> slice_start;
    std::vector<int32_t> tiles;            // [n_tiles][4] = (sequence, first q row, first position, positions)
    std::vector<int32_t> tile_base;        // first item of each tile (+1 sentinel)
    std::vector<int32_t> order;            // launch order of the items (a permutation within each slice)
    std::vector<int32_t> merge_tiles;      // tiles with more than one chunk, rising
    std::vector<int32_t> merge_start;      // first entry of merge_tiles of each merge step (+1 sentinel)
    uint64_t off_work = 0, off_tiles = 0, off_tile_base = 0, off_order = 0, off_merge_tiles = 0, off_ml = 0, off_acc = 0, upload_bytes = 0, total = 0;
  } pf;

  // pinned staging (allocated on first device use)
  void* stage = nullptr;
  size_t stage_cap = 0;
  hipEvent_t stage_ev = nullptr;
  bool stage_inflight = false;
  int32_t* remap_stage = nullptr;
  size_t remap_stage_cap = 0;
  hipEvent_t remap_ev = nullptr;
  bool remap_inflight = false;
  hipEvent_t grace_ev = nullptr;

  // slice scheduler
  // ring of events behind launches that may still be running; it persists across
  // kv_attn_run_layer calls so the host never runs more than max_inflight launches ahead
  hipEvent_t inflight_ev[vkv::kMaxInflight] = {};
  // second stream for overlapping consecutive slices of one layer (created on first use)
  bool overlap = false;
  hipStream_t aux_stream = nullptr;
  hipEvent_t fork_ev = nullptr, join_ev = nullptr;
  int inflight_head = 0, inflight_count = 0, inflight_cap = 0;
  std::atomic<int> yield_flag{0};
  // Progress words in pinned host memory that launches report to, so that the scheduler can bound
  // its lead over the GPU without an event between every two launches (an event record keeps the
  // next kernel from starting for several microseconds): word 0 = number of the newest launch that
  // has started, word 1 = number of the newest drain marker that has run.
  volatile uint32_t* progress_host = nullptr;
  uint32_t* progress_dev = nullptr;
  uint32_t launch_seq = 0;       // launches numbered so far (scheduler, one-stream mode)
  uint32_t drain_seq = 0;        // drain markers numbered so far
  uint32_t report_seq = 0;       // number the next launch_slice call reports, 0 = none
  int sched_mode = 0;            // what bounds the lead now: 0 nothing yet, 1 event ring, 2 progress words

  // per-launch timing (kv_profile_enable)
  std::vector<hipEvent_t> prof_ev;      // 2 per record: start, end
  std::vector<std::pair<int32_t, int32_t>> prof_tag;   // (kind, index)
  int32_t prof_cap = 0;
  int32_t prof_stride = 1, prof_tick = 0;   // only every prof_stride-th launch is bracketed
  std::mutex prof_mu;                  // the decode thread and the reclaim thread may both record

  bool broken = false;   // a HIP call failed mid-operation
};

namespace vkv {

bool in_released(const vkv_pool* p, int32_t b);
int  ensure_stage(vkv_pool* p, size_t bytes);
int  ensure_remap_stage(vkv_pool* p);

// Brackets one kernel launch with timing events while recording is on.
struct ProfScope {
  vkv_pool* p;
  hipStream_t st;
  int slot = -1;
  ProfScope(vkv_pool* pool, int32_t kind, int32_t index, hipStream_t stream) : p(pool), st(stream) {
    if (p->prof_cap > 0) {
      std::lock_guard<std::mutex> g(p->prof_mu);
      // sampling thins out the many slice launches; the few other launches are always bracketed
      const bool many = kind == VKV_PROF_SLICE || kind == VKV_PROF_PREFILL;
      if ((!many || p->prof_tick++ % p->prof_stride == 0) && (int32_t)p->prof_tag.size() < p->prof_cap) {
        slot = (int)p->prof_tag.size();
        p->prof_tag.emplace_back(kind, index);
      }
    }
    if (slot >= 0) (void)hipEventRecord(p->prof_ev[2 * slot], st);
  }
  ~ProfScope() {
    if (slot >= 0) (void)hipEventRecord(p->prof_ev[2 * slot + 1], st);
  }
};

// Timing of a single kernel launch while recording is on: the launch itself carries the two events
// (they take the dispatch's own start and end times), so nothing is enqueued between this kernel and
// its neighbours and the figure is the kernel's duration alone.
struct ProfKernel {
  vkv_pool* p;
  int slot = -1;
  ProfKernel(vkv_pool* pool, int32_t kind, int32_t index) : p(pool) {
    if (p->prof_cap > 0) {
      std::lock_guard<std::mutex> g(p->prof_mu);
      if (p->prof_tick++ % p->prof_stride == 0 && (int32_t)p->prof_tag.size() < p->prof_cap) {
        slot = (int)p->prof_tag.size();
        p->prof_tag.emplace_back(kind, index);
      }
    }
  }
  template <typename K, typename... Args>
  void launch(K kernel, dim3 grid, dim3 block, hipStream_t st, Args... args) {
    if (slot >= 0)
      hipExtLaunchKernelGGL(kernel, grid, block, 0, st, p->prof_ev[2 * slot], p->prof_ev[2 * slot + 1], 0, args...);
    else
      hipLaunchKernelGGL(kernel, grid, block, 0, st, args...);
  }
};

// Device address of the library's static scratch array on the current device (attn.hip);
// the first call on a device looks it up.
int static_scratch_for_current_device(void** out);

// Slice scheduler shared by decode and prefill (attn.hip).
// true if handles [first, last) of the arena all have physical memory behind them
bool arena_range_mapped(const vkv_arena* a, int32_t first, int32_t last);
int run_slices(vkv_pool* p, int32_t* cursor, int32_t n_slices, int32_t max_inflight, hipStream_t hs, const char* who,
               const std::function<int(int32_t, hipStream_t)>& launch, int32_t n_tail,
               const std::function<int(int32_t)>& tail, bool launches_report,
               const std::function<int()>& after_slices = nullptr);
int ensure_progress_words(vkv_pool* p);

// Algorithm 1 on the host tables; evicted[r] != 0 for the requests that go.  See kv_select_handles.
int select_handles_impl(const vkv_pool* p, const int32_t* tables, int32_t n_rows, int32_t max_blk, const int64_t* cost,
                        int32_t k, int32_t* handles_out, std::vector<uint8_t>& evicted, int64_t* total_out, const char* who);
// Waits until work enqueued so far on `ds` (if it differs from `cs`) and on the pool's second stream
// has finished: slices launched before a table rewrite may still hold old entries.
int grace_wait(vkv_pool* p, hipStream_t cs, hipStream_t ds);
int launch_rewrite(vkv_pool* p, int32_t* tables, int64_t n, const int32_t* remap, int32_t nb, hipStream_t st);

// Host-side relocation plan; see kv_reclaim_plan.
int plan_relocation(const vkv_pool* p, int32_t lo, int32_t hi,
                    std::vector<int32_t>& src, std::vector<int32_t>& dst);

}  // namespace vkv
