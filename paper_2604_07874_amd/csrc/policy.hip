// Host-side policies of the paper that steer the hot path: which handles to give up when
// relocation cannot fit (Algorithm 1, Section 5), how much headroom to keep for the online
// tenant (MIAD reservation, Section 5), and when offline work may wake up again
// (cooldown T_cool = 2G, Section 4.2).  No device work.
#include "vkv_internal.h"

#include <algorithm>
#include <cmath>
#include <deque>

using namespace vkv;

struct vkv_miad {
  vkv_miad_config c;
  int32_t h;
  double t;
  std::deque<double> events;
  bool started = false;
  double last_release = 0.0;
};

struct vkv_gate {
  double g;
  bool busy = false;
  double idle_since = 0.0;
  bool offline_on = true;
  bool has_last = false;
  int64_t last_request = 0;
  int64_t preemptions = 0;
};

// Reqs(h) as sorted, duplicate-free row lists
static void handle_rows(const vkv_pool* p, const int32_t* tables, int32_t n_rows, int32_t max_blk,
                        std::vector<std::vector<int32_t>>& reqs) {
  const int32_t bph = p->cfg.blocks_per_handle, nb = p->cfg.num_blocks;
  reqs.assign((size_t)(nb / bph), {});
  for (int32_t r = 0; r < n_rows; ++r)
    for (int32_t j = 0; j < max_blk; ++j) {
      const int32_t e = tables[(size_t)r * max_blk + j];
      if (e < 0 || e >= nb) continue;
      auto& v = reqs[(size_t)(e / bph)];
      if (v.empty() || v.back() != r) v.push_back(r);   // rows are visited in ascending order
    }
}

namespace vkv {

int select_handles_impl(const vkv_pool* p, const int32_t* tables, int32_t n_rows, int32_t max_blk, const int64_t* cost,
                        int32_t k, int32_t* handles_out, std::vector<uint8_t>& evicted, int64_t* total_out, const char* who) {
  const int32_t bph = p->cfg.blocks_per_handle, n_handles = p->cfg.num_blocks / bph;
  std::vector<std::vector<int32_t>> reqs;
  handle_rows(p, tables, n_rows, max_blk, reqs);
  std::vector<uint8_t> candidate((size_t)n_handles, 1);
  evicted.assign((size_t)n_rows, 0);
  int32_t n_cand = 0;
  for (int32_t h = 0; h < n_handles; ++h) {
    if (in_released(p, h * bph)) candidate[(size_t)h] = 0;   // already with the online tenant
    n_cand += candidate[(size_t)h];
  }
  if (k > n_cand) {
    set_error("%s: %d handles wanted, %d not yet handed over", who, k, n_cand);
    return VKV_E_NOSPACE;
  }
  // Cost of a handle = summed cost of its requests not yet evicted.  Kept up to date as requests go
  // (the same integers a fresh sum would give), so that a pick is one pass over the handles.
  std::vector<std::vector<int32_t>> row_handles((size_t)n_rows);
  std::vector<int64_t> hcost((size_t)n_handles, 0);
  for (int32_t h = 0; h < n_handles; ++h)
    for (int32_t r : reqs[(size_t)h]) {
      row_handles[(size_t)r].push_back(h);
      hcost[(size_t)h] += cost[r];
    }
  int64_t total = 0;
  for (int32_t i = 0; i < k; ++i) {
    int32_t best = -1;
    for (int32_t h = 0; h < n_handles; ++h)
      if (candidate[(size_t)h] && (best < 0 || hcost[(size_t)h] < hcost[(size_t)best])) best = h;   // ties: lowest index
    handles_out[i] = best;
    candidate[(size_t)best] = 0;
    total += hcost[(size_t)best];
    for (int32_t r : reqs[(size_t)best]) {
      if (evicted[(size_t)r]) continue;
      evicted[(size_t)r] = 1;
      for (int32_t h : row_handles[(size_t)r]) hcost[(size_t)h] -= cost[r];
    }
  }
  if (total_out) *total_out = total;
  return VKV_OK;
}

// one row of a device block table per workgroup: every entry becomes -1
__global__ __launch_bounds__(256) void table_clear_rows_kernel(int32_t* __restrict__ tables, int32_t max_blk,
                                                                const int32_t* __restrict__ rows) {
  int32_t* row = tables + (size_t)rows[blockIdx.x] * max_blk;
  for (int32_t j = threadIdx.x; j < max_blk; j += blockDim.x) row[j] = -1;
}

}  // namespace vkv

static bool bad_tables(int32_t n_rows, int32_t max_blk, const int32_t* tables) {
  return n_rows < 0 || max_blk < 0 || (n_rows > 0 && max_blk > 0 && !tables);
}

// Entries of the host tables that name a block of a chosen handle, row-major; count only when the outputs are NULL.
static int64_t list_invalidated(const vkv_pool* p, const std::vector<uint8_t>& chosen, const int32_t* tables, int32_t n_rows,
                                int32_t max_blk, int32_t* rows, int32_t* cols, int32_t* blks) {
  const int32_t bph = p->cfg.blocks_per_handle;
  int64_t n = 0;
  for (int32_t r = 0; r < n_rows; ++r)
    for (int32_t j = 0; j < max_blk; ++j) {
      const int32_t e = tables[(size_t)r * max_blk + j];
      if (e >= 0 && e < p->cfg.num_blocks && chosen[(size_t)(e / bph)]) {
        if (rows) rows[n] = r;
        if (cols) cols[n] = j;
        if (blks) blks[n] = e;
        ++n;
      }
    }
  return n;
}

extern "C" {

int kv_select_handles(vkv_pool* p, const int32_t* tables, int32_t n_rows, int32_t max_blk, const int64_t* cost,
                      int32_t k, int32_t* handles_out, int32_t* evicted_rows_out, int32_t* n_evicted_out,
                      int64_t* total_cost_out) {
  if (!p || bad_tables(n_rows, max_blk, tables) || (n_rows > 0 && !cost) || k < 0 || (k > 0 && !handles_out)) {
    set_error("kv_select_handles: bad argument");
    return VKV_E_INVAL;
  }
  std::vector<uint8_t> evicted;
  int st = select_handles_impl(p, tables, n_rows, max_blk, cost, k, handles_out, evicted, total_cost_out, "kv_select_handles");
  if (st != VKV_OK) return st;
  int32_t n_ev = 0;
  for (int32_t r = 0; r < n_rows; ++r)
    if (evicted[(size_t)r]) {
      if (evicted_rows_out) evicted_rows_out[n_ev] = r;
      ++n_ev;
    }
  if (n_evicted_out) *n_evicted_out = n_ev;
  return VKV_OK;
}

int kv_handles_cost(vkv_pool* p, const int32_t* tables, int32_t n_rows, int32_t max_blk, const int64_t* cost,
                    const int32_t* handles, int32_t k, int32_t* evicted_rows_out, int32_t* n_evicted_out,
                    int64_t* total_cost_out) {
  if (!p || bad_tables(n_rows, max_blk, tables) || (n_rows > 0 && !cost) || k < 0 || (k > 0 && !handles)) {
    set_error("kv_handles_cost: bad argument");
    return VKV_E_INVAL;
  }
  const int32_t bph = p->cfg.blocks_per_handle, n_handles = p->cfg.num_blocks / bph;
  std::vector<uint8_t> chosen((size_t)n_handles, 0);
  for (int32_t i = 0; i < k; ++i) {
    if (handles[i] < 0 || handles[i] >= n_handles) { set_error("kv_handles_cost: bad handle %d", handles[i]); return VKV_E_INVAL; }
    chosen[(size_t)handles[i]] = 1;
  }
  int32_t n_ev = 0;
  int64_t total = 0;
  for (int32_t r = 0; r < n_rows; ++r) {
    bool hit = false;
    for (int32_t j = 0; j < max_blk && !hit; ++j) {
      const int32_t e = tables[(size_t)r * max_blk + j];
      hit = e >= 0 && e < p->cfg.num_blocks && chosen[(size_t)(e / bph)];
    }
    if (hit) {
      if (evicted_rows_out) evicted_rows_out[n_ev] = r;
      ++n_ev;
      total += cost[r];
    }
  }
  if (n_evicted_out) *n_evicted_out = n_ev;
  if (total_cost_out) *total_cost_out = total;
  return VKV_OK;
}

int kv_invalidate_handles(vkv_pool* p, const int32_t* handles, int32_t k, const int32_t* tables, int32_t n_rows,
                          int32_t max_blk, int32_t* inv_row_out, int32_t* inv_col_out, int32_t* inv_block_out,
                          int32_t cap, int32_t* n_inv_out, int32_t* tables_dev, int32_t* remap_dev, void* stream_v,
                          void* decode_stream_v) {
  if (!p || k < 0 || (k > 0 && !handles) || bad_tables(n_rows, max_blk, tables) || cap < 0 || !n_inv_out ||
      (tables_dev && !remap_dev)) {
    set_error("kv_invalidate_handles: bad argument");
    return VKV_E_INVAL;
  }
  if (tables_dev && p->broken) { set_error("kv_invalidate_handles: pool unusable after a HIP failure"); return VKV_E_HIP; }
  const int32_t bph = p->cfg.blocks_per_handle, n_handles = p->cfg.num_blocks / bph, nb = p->cfg.num_blocks;
  std::vector<uint8_t> chosen((size_t)n_handles, 0);
  for (int32_t i = 0; i < k; ++i) {
    const int32_t h = handles[i];
    if (h < 0 || h >= n_handles || chosen[(size_t)h]) { set_error("kv_invalidate_handles: bad or repeated handle %d", h); return VKV_E_INVAL; }
    if (in_released(p, h * bph)) { set_error("kv_invalidate_handles: handle %d is already handed over", h); return VKV_E_BUSY; }
    chosen[(size_t)h] = 1;
  }
  // count first, so that a too small output leaves everything untouched
  const int64_t n_inv = list_invalidated(p, chosen, tables, n_rows, max_blk, nullptr, nullptr, nullptr);
  if (n_inv > cap) {
    *n_inv_out = (int32_t)std::min<int64_t>(n_inv, 0x7FFFFFFF);
    set_error("kv_invalidate_handles: %lld invalidated entries, room for %d", (long long)n_inv, cap);
    return VKV_E_NOSPACE;
  }
  if (tables_dev) {
    // The device tables lose the entries too (they become -1, which the kernels skip and flag), and the
    // slices that may still hold the old entries are waited for: from then on nothing reads the handles.
    hipStream_t cs = (hipStream_t)stream_v;
    int st = ensure_remap_stage(p);
    if (st != VKV_OK) return st;
    for (int32_t b = 0; b < nb; ++b) p->remap_stage[b] = chosen[(size_t)(b / bph)] ? -1 : b;
    auto fail = [&](int code) { p->broken = true; return code; };
    hipError_t he = hipMemcpyAsync(remap_dev, p->remap_stage, (size_t)nb * 4, hipMemcpyHostToDevice, cs);
    if (he != hipSuccess) return fail(hip_fail(he, "remap upload"));
    if (launch_rewrite(p, tables_dev, (int64_t)n_rows * max_blk, remap_dev, nb, cs) != VKV_OK) return fail(VKV_E_HIP);
    he = hipStreamSynchronize(cs);
    if (he != hipSuccess) return fail(hip_fail(he, "hipStreamSynchronize"));
    if (grace_wait(p, cs, (hipStream_t)decode_stream_v) != VKV_OK) return fail(VKV_E_HIP);
  }
  *n_inv_out = (int32_t)list_invalidated(p, chosen, tables, n_rows, max_blk, inv_row_out, inv_col_out, inv_block_out);
  for (int32_t h = 0; h < n_handles; ++h) {
    if (!chosen[(size_t)h]) continue;
    for (int32_t b = h * bph; b < (h + 1) * bph; ++b)
      if (p->live[(size_t)b]) { p->live[(size_t)b] = 0; --p->n_live; }
  }
  for (int32_t i = 0; i < k; ++i)   // in the order given
    p->hand_over(handles[i] * bph, (handles[i] + 1) * bph, tables_dev != nullptr);
  return VKV_OK;
}

int kv_evict_handles(vkv_pool* p, int32_t k, int32_t* tables, int32_t n_rows, int32_t max_blk, const int64_t* cost,
                     int32_t* tables_dev, int32_t* scratch_dev, void* stream_v, void* decode_stream_v,
                     int32_t* handles_out, int32_t* evicted_rows_out, int32_t* inv_row_out, int32_t* inv_col_out,
                     int32_t* inv_block_out, int32_t cap, vkv_evict_info* info) {
  if (!p || k < 0 || (k > 0 && !handles_out) || bad_tables(n_rows, max_blk, tables) || (n_rows > 0 && !cost) || cap < 0 ||
      !info || (tables_dev && !scratch_dev)) {
    set_error("kv_evict_handles: bad argument");
    return VKV_E_INVAL;
  }
  if (tables_dev && p->broken) { set_error("kv_evict_handles: pool unusable after a HIP failure"); return VKV_E_HIP; }
  const int32_t bph = p->cfg.blocks_per_handle, n_handles = p->cfg.num_blocks / bph, nb = p->cfg.num_blocks;
  if (tables_dev && n_rows > nb) { set_error("kv_evict_handles: more table rows than blocks"); return VKV_E_INVAL; }
  std::vector<uint8_t> evicted;
  int64_t total = 0;
  int st = select_handles_impl(p, tables, n_rows, max_blk, cost, k, handles_out, evicted, &total, "kv_evict_handles");
  if (st != VKV_OK) return st;
  std::vector<uint8_t> chosen((size_t)n_handles, 0);
  for (int32_t i = 0; i < k; ++i) chosen[(size_t)handles_out[i]] = 1;
  const int64_t n_inv = list_invalidated(p, chosen, tables, n_rows, max_blk, nullptr, nullptr, nullptr);
  *info = vkv_evict_info{};
  info->n_invalidated = (int32_t)std::min<int64_t>(n_inv, 0x7FFFFFFF);
  if (n_inv > cap) {
    set_error("kv_evict_handles: %lld invalidated entries, room for %d", (long long)n_inv, cap);
    return VKV_E_NOSPACE;
  }
  std::vector<int32_t> rows;
  for (int32_t r = 0; r < n_rows; ++r)
    if (evicted[(size_t)r]) rows.push_back(r);
  if (tables_dev && !rows.empty()) {
    // Every request with a block in a chosen handle goes whole, so clearing their rows leaves no entry
    // that names a chosen handle.  Then the slices that may still hold old entries are waited for.
    hipStream_t cs = (hipStream_t)stream_v;
    st = ensure_remap_stage(p);
    if (st != VKV_OK) return st;
    std::copy(rows.begin(), rows.end(), p->remap_stage);
    auto fail = [&](int code) { p->broken = true; return code; };
    hipError_t he = hipMemcpyAsync(scratch_dev, p->remap_stage, rows.size() * 4, hipMemcpyHostToDevice, cs);
    if (he != hipSuccess) return fail(hip_fail(he, "row list upload"));
    hipLaunchKernelGGL(table_clear_rows_kernel, dim3((unsigned)rows.size()), dim3(256), 0, cs, tables_dev, max_blk,
                       (const int32_t*)scratch_dev);
    he = hipGetLastError();
    if (he != hipSuccess) return fail(hip_fail(he, "table_clear_rows launch"));
    he = hipStreamSynchronize(cs);
    if (he != hipSuccess) return fail(hip_fail(he, "hipStreamSynchronize"));
    if (grace_wait(p, cs, (hipStream_t)decode_stream_v) != VKV_OK) return fail(VKV_E_HIP);
  }
  list_invalidated(p, chosen, tables, n_rows, max_blk, inv_row_out, inv_col_out, inv_block_out);
  // blocks the survivors still name stay live whatever row else named them
  std::vector<uint8_t> kept((size_t)nb, 0);
  for (int32_t r = 0; r < n_rows; ++r) {
    if (evicted[(size_t)r]) continue;
    for (int32_t j = 0; j < max_blk; ++j) {
      const int32_t e = tables[(size_t)r * max_blk + j];
      if (e >= 0 && e < nb) kept[(size_t)e] = 1;
    }
  }
  for (int32_t r : rows)
    for (int32_t j = 0; j < max_blk; ++j) {
      int32_t& e = tables[(size_t)r * max_blk + j];
      if (e >= 0 && e < nb && !kept[(size_t)e] && p->live[(size_t)e]) { p->live[(size_t)e] = 0; --p->n_live; }
      e = -1;
    }
  for (int32_t i = 0; i < k; ++i) {
    const int32_t h = handles_out[i];
    for (int32_t b = h * bph; b < (h + 1) * bph; ++b)
      if (p->live[(size_t)b]) { p->live[(size_t)b] = 0; --p->n_live; }
    p->hand_over(h * bph, (h + 1) * bph, tables_dev != nullptr || rows.empty());
  }
  if (evicted_rows_out) std::copy(rows.begin(), rows.end(), evicted_rows_out);
  info->mode = 1;
  info->n_handles = k;
  info->n_evicted = (int32_t)rows.size();
  info->total_cost = total;
  return VKV_OK;
}

int kv_reclaim_or_evict(vkv_pool* p, int32_t lo, int32_t hi, int32_t* tables_dev, int32_t* tables, int32_t n_rows,
                        int32_t max_blk, const int64_t* cost, uint64_t chunk_bytes, uint64_t rate_cap, void* copy_stream,
                        void* decode_stream, int32_t* remap_dev, uint32_t flags, int32_t* handles_out,
                        int32_t* evicted_rows_out, int32_t* inv_row_out, int32_t* inv_col_out, int32_t* inv_block_out,
                        int32_t cap, vkv_evict_info* info, vkv_reclaim_stats* stats) {
  if (!p || !info || bad_tables(n_rows, max_blk, tables) || !tables_dev) {
    set_error("kv_reclaim_or_evict: bad argument");
    return VKV_E_INVAL;
  }
  *info = vkv_evict_info{};
  int st = kv_reclaim_range(p, lo, hi, tables_dev, (int64_t)n_rows * max_blk, chunk_bytes, rate_cap, copy_stream,
                            decode_stream, remap_dev, flags, stats);
  if (st == VKV_OK) {
    // the host copy of the tables follows the device's: the remap of this call is in the pinned staging
    // buffer (the upload has finished unless the call was asynchronous, and the host wrote it anyway)
    const int32_t nb = p->cfg.num_blocks;
    for (int64_t i = 0; i < (int64_t)n_rows * max_blk; ++i)
      if (tables[i] >= 0 && tables[i] < nb) tables[i] = p->remap_stage[tables[i]];
    return VKV_OK;
  }
  if (st != VKV_E_NOSPACE) return st;
  const int32_t k = (hi - lo) / p->cfg.blocks_per_handle;
  return kv_evict_handles(p, k, tables, n_rows, max_blk, cost, tables_dev, remap_dev, copy_stream, decode_stream,
                          handles_out, evicted_rows_out, inv_row_out, inv_col_out, inv_block_out, cap, info);
}

// ---- MIAD headroom ----------------------------------------------------------------------

int kv_miad_init(const vkv_miad_config* c, vkv_miad** out) {
  if (!c || !out) { set_error("kv_miad_init: null argument"); return VKV_E_INVAL; }
  *out = nullptr;
  if (c->h_min < 1 || c->h_init < c->h_min || c->h_max < c->h_init || !(c->alpha > 1.0) ||
      !(c->pressure_frac > 0.0 && c->pressure_frac <= 1.0) || !(c->t_min > 0.0) || c->t_init < c->t_min ||
      c->t_max < c->t_init || !(c->t_up > 1.0) || c->t_down < 0.0 || !(c->window_s > 0.0) || c->target_rate < 0.0) {
    set_error("kv_miad_init: inconsistent configuration");
    return VKV_E_INVAL;
  }
  vkv_miad* m = new vkv_miad();
  m->c = *c;
  m->h = c->h_init;
  m->t = c->t_init;
  *out = m;
  return VKV_OK;
}

int kv_miad_destroy(vkv_miad* m) {
  delete m;
  return VKV_OK;
}

static void adapt_interval(vkv_miad* m, double now) {
  while (!m->events.empty() && !(m->events.front() > now - m->c.window_s)) m->events.pop_front();
  const double rate = (double)m->events.size() / m->c.window_s;
  if (rate > m->c.target_rate) m->t = std::min(m->c.t_max, m->t * m->c.t_up);
  else m->t = std::max(m->c.t_min, m->t - m->c.t_down);
}

int kv_miad_observe(vkv_miad* m, double now_s, int32_t used_handles, vkv_miad_step* out) {
  if (!m || !out || used_handles < 0) { set_error("kv_miad_observe: bad argument"); return VKV_E_INVAL; }
  if (!m->started) { m->started = true; m->last_release = now_s; }
  *out = vkv_miad_step{};
  if ((double)used_handles >= m->c.pressure_frac * (double)m->h) {
    out->pressure_event = 1;
    const int32_t grown = (int32_t)std::ceil((double)m->h * m->c.alpha);
    const int32_t new_h = std::min(m->c.h_max, std::max(m->h + 1, grown));
    out->grow_by = new_h - m->h;
    m->h = new_h;
    m->events.push_back(now_s);
    adapt_interval(m, now_s);
    m->last_release = now_s;
  } else if (now_s - m->last_release >= m->t) {
    if (m->h > m->c.h_min && m->h - 1 > used_handles) {
      --m->h;
      out->release = 1;
    }
    m->last_release = now_s;
    adapt_interval(m, now_s);
  }
  out->headroom = m->h;
  out->interval_s = m->t;
  return VKV_OK;
}

// ---- cooldown gate ---------------------------------------------------------------------

int kv_gate_init(double initial_gap_s, vkv_gate** out) {
  if (!out || !(initial_gap_s >= 0.0)) { set_error("kv_gate_init: bad argument"); return VKV_E_INVAL; }
  vkv_gate* g = new vkv_gate();
  g->g = initial_gap_s;
  *out = g;
  return VKV_OK;
}

int kv_gate_destroy(vkv_gate* g) {
  delete g;
  return VKV_OK;
}

int kv_gate_online_busy(vkv_gate* g, double now_s, int64_t request_id) {
  if (!g) return VKV_E_INVAL;
  int preempt = 0;
  if (!g->busy) {
    if (g->has_last && request_id == g->last_request) g->g = std::max(g->g, now_s - g->idle_since);
    g->busy = true;
  }
  if (g->offline_on) {
    g->offline_on = false;
    ++g->preemptions;
    preempt = 1;
  }
  g->has_last = true;
  g->last_request = request_id;
  return preempt;
}

int kv_gate_online_idle(vkv_gate* g, double now_s) {
  if (!g) return VKV_E_INVAL;
  if (g->busy) {
    g->busy = false;
    g->idle_since = now_s;
  }
  return VKV_OK;
}

int kv_gate_poll(vkv_gate* g, double now_s) {
  if (!g) return VKV_E_INVAL;
  if (!g->offline_on && !g->busy && now_s - g->idle_since >= 2.0 * g->g) g->offline_on = true;
  return g->offline_on ? 1 : 0;
}

int kv_gate_stats(vkv_gate* g, double* max_gap_s_out, int64_t* preemptions_out) {
  if (!g) return VKV_E_INVAL;
  if (max_gap_s_out) *max_gap_s_out = g->g;
  if (preemptions_out) *preemptions_out = g->preemptions;
  return VKV_OK;
}

}  // extern "C"
