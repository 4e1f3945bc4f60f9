// Pool bookkeeping: geometry, occupancy bitmap, handed-over ranges, allocate-release
// interface (paper Section 3: a global pool of coarse equal-size handles shared
// through allocate/release).  Host only.
#include "vkv_internal.h"

#include <algorithm>
#include <cstring>

namespace vkv {

static thread_local std::string g_err;

void set_error(const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
}

int hip_fail(hipError_t e, const char* what) {
  set_error("HIP error %d (%s) in %s", (int)e, hipGetErrorString(e), what);
  return VKV_E_HIP;
}

bool in_released(const vkv_pool* p, int32_t b) { return p->handed[(size_t)b] != 0; }

int ensure_stage(vkv_pool* p, size_t bytes) {
  if (!p->stage_ev) VKV_HIP(hipEventCreateWithFlags(&p->stage_ev, hipEventDisableTiming));
  if (p->stage_inflight) {
    VKV_HIP(hipEventSynchronize(p->stage_ev));
    p->stage_inflight = false;
  }
  if (p->stage_cap < bytes) {
    if (p->stage) VKV_HIP(hipHostFree(p->stage));
    p->stage = nullptr;
    p->stage_cap = 0;
    size_t cap = std::max<size_t>(bytes * 2, 1 << 16);
    VKV_HIP(hipHostMalloc(&p->stage, cap, hipHostMallocDefault));
    p->stage_cap = cap;
  }
  return VKV_OK;
}

int ensure_remap_stage(vkv_pool* p) {
  if (!p->remap_ev) VKV_HIP(hipEventCreateWithFlags(&p->remap_ev, hipEventDisableTiming));
  if (!p->grace_ev) VKV_HIP(hipEventCreateWithFlags(&p->grace_ev, hipEventDisableTiming));
  if (p->remap_inflight) {
    VKV_HIP(hipEventSynchronize(p->remap_ev));
    p->remap_inflight = false;
  }
  size_t need = (size_t)p->cfg.num_blocks * sizeof(int32_t);
  if (p->remap_stage_cap < need) {
    void* m = nullptr;
    VKV_HIP(hipHostMalloc(&m, need, hipHostMallocDefault));
    p->remap_stage = (int32_t*)m;
    p->remap_stage_cap = need;
  }
  return VKV_OK;
}

}  // namespace vkv

using namespace vkv;

extern "C" {

const char* vkv_last_error(void) { return g_err.c_str(); }

int kv_pool_init(const vkv_pool_config* c, vkv_pool** out) {
  if (!c || !out) { set_error("kv_pool_init: null argument"); return VKV_E_INVAL; }
  *out = nullptr;
  if (c->num_layers < 1 || c->num_q_heads < 1 || c->num_kv_heads < 1 || c->num_blocks < 1 ||
      c->blocks_per_handle < 1) {
    set_error("kv_pool_init: counts must be positive");
    return VKV_E_INVAL;
  }
  if (c->num_q_heads % c->num_kv_heads || c->num_q_heads / c->num_kv_heads > 16) {
    set_error("kv_pool_init: num_q_heads must be a multiple (at most 16x) of num_kv_heads");
    return VKV_E_INVAL;
  }
  if (c->head_dim != 64 && c->head_dim != 128) {
    set_error("kv_pool_init: head_dim must be 64 or 128");
    return VKV_E_INVAL;
  }
  if (c->block_tokens != 16) { set_error("kv_pool_init: block_tokens must be 16"); return VKV_E_INVAL; }
  if (c->num_blocks % c->blocks_per_handle) {
    set_error("kv_pool_init: num_blocks must be a multiple of blocks_per_handle");
    return VKV_E_INVAL;
  }
  uint64_t be = (uint64_t)c->num_layers * 2 * c->num_kv_heads * c->block_tokens * c->head_dim;
  if (c->base) {
    if ((uintptr_t)c->base % 16) { set_error("kv_pool_init: base must be 16-byte aligned"); return VKV_E_INVAL; }
    if (c->bytes < be * 2 * (uint64_t)c->num_blocks) {
      set_error("kv_pool_init: %llu bytes given, %llu needed", (unsigned long long)c->bytes,
                (unsigned long long)(be * 2 * (uint64_t)c->num_blocks));
      return VKV_E_INVAL;
    }
  }
  vkv_pool* p = new vkv_pool();
  p->cfg = *c;
  p->G = c->num_q_heads / c->num_kv_heads;
  p->block_elems = be;
  p->block_bytes = be * 2;
  p->live.assign((size_t)c->num_blocks, 0);
  p->handed.assign((size_t)c->num_blocks, 0);
  if (c->base) {
    // a pool with device memory: find this device's copy of the static scratch now, so that
    // paged_decode_attn_layer_static has nothing left to set up (a failure here is reported there)
    void* scratch = nullptr;
    (void)static_scratch_for_current_device(&scratch);
  }
  *out = p;
  return VKV_OK;
}

int kv_pool_destroy(vkv_pool* p) {
  if (!p) return VKV_OK;
  // Best effort: report nothing, the process may be shutting the runtime down.
  if (p->stage) (void)hipHostFree(p->stage);
  if (p->remap_stage) (void)hipHostFree(p->remap_stage);
  if (p->progress_host) (void)hipHostFree((void*)p->progress_host);
  if (p->stage_ev) (void)hipEventDestroy(p->stage_ev);
  if (p->remap_ev) (void)hipEventDestroy(p->remap_ev);
  if (p->grace_ev) (void)hipEventDestroy(p->grace_ev);
  if (p->fork_ev) (void)hipEventDestroy(p->fork_ev);
  if (p->join_ev) (void)hipEventDestroy(p->join_ev);
  if (p->aux_stream) (void)hipStreamDestroy(p->aux_stream);
  for (auto& e : p->inflight_ev)
    if (e) (void)hipEventDestroy(e);
  for (auto& e : p->prof_ev) (void)hipEventDestroy(e);
  delete p;
  return VKV_OK;
}

int kv_pool_alloc(vkv_pool* p, int32_t n, int32_t* ids) {
  if (!p || n < 0 || (n > 0 && !ids)) { set_error("kv_pool_alloc: bad argument"); return VKV_E_INVAL; }
  std::vector<int32_t> got;
  got.reserve((size_t)n);
  for (int32_t b = 0; b < p->cfg.num_blocks && (int32_t)got.size() < n; ++b)
    if (!p->live[b] && !in_released(p, b)) got.push_back(b);
  if ((int32_t)got.size() < n) {
    set_error("kv_pool_alloc: %d blocks wanted, %d free", n, (int)got.size());
    return VKV_E_NOSPACE;
  }
  for (int32_t b : got) p->live[b] = 1;
  p->n_live += n;
  std::copy(got.begin(), got.end(), ids);
  return VKV_OK;
}

static int check_ids(vkv_pool* p, const int32_t* ids, int32_t n, uint8_t want_live, const char* who) {
  if (!p || n < 0 || (n > 0 && !ids)) { set_error("%s: bad argument", who); return VKV_E_INVAL; }
  std::vector<int32_t> sorted(ids, ids + n);
  std::sort(sorted.begin(), sorted.end());
  for (int32_t i = 0; i < n; ++i) {
    int32_t b = sorted[i];
    if (b < 0 || b >= p->cfg.num_blocks) { set_error("%s: block %d out of range", who, b); return VKV_E_INVAL; }
    if (i && sorted[i - 1] == b) { set_error("%s: block %d listed twice", who, b); return VKV_E_INVAL; }
    if (p->live[b] != want_live) {
      set_error("%s: block %d is %s", who, b, want_live ? "not live" : "already live");
      return VKV_E_INVAL;
    }
    if (!want_live && in_released(p, b)) {
      set_error("%s: block %d lies in a handed-over range", who, b);
      return VKV_E_INVAL;
    }
  }
  return VKV_OK;
}

int kv_pool_adopt(vkv_pool* p, const int32_t* ids, int32_t n) {
  int st = check_ids(p, ids, n, 0, "kv_pool_adopt");
  if (st != VKV_OK) return st;
  for (int32_t i = 0; i < n; ++i) p->live[ids[i]] = 1;
  p->n_live += n;
  return VKV_OK;
}

int kv_pool_free(vkv_pool* p, const int32_t* ids, int32_t n) {
  int st = check_ids(p, ids, n, 1, "kv_pool_free");
  if (st != VKV_OK) return st;
  for (int32_t i = 0; i < n; ++i) p->live[ids[i]] = 0;
  p->n_live -= n;
  return VKV_OK;
}

int kv_pool_return_range(vkv_pool* p, int32_t lo, int32_t hi) {
  if (!p) { set_error("kv_pool_return_range: null pool"); return VKV_E_INVAL; }
  const int32_t bph = p->cfg.blocks_per_handle;
  if (lo < 0 || hi > p->cfg.num_blocks || lo >= hi || lo % bph || hi % bph) {
    set_error("kv_pool_return_range: [%d,%d) must be non-empty, inside the pool and a multiple of %d blocks", lo, hi, bph);
    return VKV_E_INVAL;
  }
  for (size_t i = 0; i < p->released.size(); ++i) {
    const vkv_pool::Range r = p->released[i];
    if (r.first <= lo && hi <= r.second) {
      if (p->arena && !arena_range_mapped(p->arena, lo / bph, hi / bph)) {
        set_error("kv_pool_return_range: handles of [%d,%d) are unmapped; kv_arena_restore first", lo, hi);
        return VKV_E_STATE;
      }
      // what is left of the range on either side stays handed over
      p->released.erase(p->released.begin() + (long)i);
      std::fill(p->handed.begin() + lo, p->handed.begin() + hi, (uint8_t)0);
      if (hi < r.second) p->released.insert(p->released.begin() + (long)i, vkv_pool::Range(hi, r.second, r.clean));
      if (r.first < lo) p->released.insert(p->released.begin() + (long)i, vkv_pool::Range(r.first, lo, r.clean));
      return VKV_OK;
    }
  }
  set_error("kv_pool_return_range: [%d,%d) does not lie inside one handed-over range", lo, hi);
  return VKV_E_INVAL;
}

int kv_pool_state(vkv_pool* p, uint8_t* live_out, int32_t* ranges_out, int32_t cap, int32_t* n_ranges) {
  if (!p) { set_error("kv_pool_state: null pool"); return VKV_E_INVAL; }
  if (live_out) std::memcpy(live_out, p->live.data(), p->live.size());
  if (n_ranges) *n_ranges = (int32_t)p->released.size();
  if (ranges_out) {
    for (int32_t i = 0; i < cap && i < (int32_t)p->released.size(); ++i) {
      ranges_out[2 * i] = p->released[i].first;
      ranges_out[2 * i + 1] = p->released[i].second;
    }
  }
  return VKV_OK;
}

int kv_pool_check_tables(vkv_pool* p, const int32_t* t, int64_t n) {
  if (!p || (n > 0 && !t) || n < 0) { set_error("kv_pool_check_tables: bad argument"); return VKV_E_INVAL; }
  for (int64_t i = 0; i < n; ++i) {
    int32_t e = t[i];
    if (e == -1) continue;
    if (e < 0 || e >= p->cfg.num_blocks) {
      set_error("table entry %lld = %d is outside the pool", (long long)i, e);
      return VKV_E_STATE;
    }
    if (!p->live[e]) { set_error("table entry %lld names block %d, which is not live", (long long)i, e); return VKV_E_STATE; }
    if (in_released(p, e)) {
      set_error("table entry %lld names block %d inside a handed-over range", (long long)i, e);
      return VKV_E_STATE;
    }
  }
  return VKV_OK;
}

int kv_profile_enable(vkv_pool* p, int32_t max_records) {
  if (!p || max_records < 0 || max_records > (1 << 20)) { set_error("kv_profile_enable: bad argument"); return VKV_E_INVAL; }
  for (auto& e : p->prof_ev) (void)hipEventDestroy(e);
  p->prof_ev.clear();
  p->prof_tag.clear();
  p->prof_cap = 0;
  p->prof_ev.reserve((size_t)max_records * 2);
  p->prof_tag.reserve((size_t)max_records);
  for (int32_t i = 0; i < 2 * max_records; ++i) {
    hipEvent_t e = nullptr;
    VKV_HIP(hipEventCreate(&e));
    p->prof_ev.push_back(e);
  }
  p->prof_cap = max_records;
  return VKV_OK;
}

int kv_profile_sample(vkv_pool* p, int32_t stride) {
  if (!p || stride < 1) { set_error("kv_profile_sample: need a pool and stride >= 1"); return VKV_E_INVAL; }
  std::lock_guard<std::mutex> g(p->prof_mu);
  p->prof_stride = stride;
  p->prof_tick = 0;
  return VKV_OK;
}

int kv_profile_read(vkv_pool* p, vkv_profile_record* out, int32_t cap, int32_t* n_out) {
  if (!p || cap < 0 || (cap > 0 && !out) || !n_out) { set_error("kv_profile_read: bad argument"); return VKV_E_INVAL; }
  const int32_t n = std::min<int32_t>(cap, (int32_t)p->prof_tag.size());
  for (int32_t i = 0; i < n; ++i) {
    VKV_HIP(hipEventSynchronize(p->prof_ev[2 * i + 1]));
    float ms = 0.f;
    VKV_HIP(hipEventElapsedTime(&ms, p->prof_ev[2 * i], p->prof_ev[2 * i + 1]));
    out[i].kind = p->prof_tag[i].first;
    out[i].index = p->prof_tag[i].second;
    out[i].ms = ms;
  }
  if (!p->prof_tag.empty()) VKV_HIP(hipEventSynchronize(p->prof_ev[2 * p->prof_tag.size() - 1]));
  *n_out = n;
  p->prof_tag.clear();
  return VKV_OK;
}

int kv_yield_request(vkv_pool* p) {
  if (!p) return VKV_E_INVAL;
  p->yield_flag.store(1, std::memory_order_release);
  return VKV_OK;
}
int kv_yield_clear(vkv_pool* p) {
  if (!p) return VKV_E_INVAL;
  p->yield_flag.store(0, std::memory_order_release);
  return VKV_OK;
}
int kv_yield_pending(vkv_pool* p) { return p ? p->yield_flag.load(std::memory_order_acquire) : 0; }

}  // extern "C"
