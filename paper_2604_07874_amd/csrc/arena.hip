// Handle-backed pool memory: one reservation of device address space, one physical allocation
// per handle (HIP virtual-memory API).  The paper's KV memory is allocated and released in
// equal-size handles, and a reclaimed handle goes back to the online tenant for good
// (Section 5).  With the pool's memory laid out this way, a range that kv_reclaim_range has
// emptied and handed over can be unmapped and its physical memory returned to the driver, so
// that any other allocation on the device (another process included) can have it; when the
// online tenant gives the range back, fresh physical memory is mapped at the same addresses and
// no block id or table entry changes.
//
// Unmapping is safe only for memory nothing will touch.  The calls here therefore check the pool's
// own record: a handle is unmapped only while its blocks are inside a handed-over range, which
// kv_reclaim_range enters after the copy, the table rewrite and the grace wait, and which the
// allocator, the relocation planner and every block table then avoid.
#include "vkv_internal.h"

#include <vector>

struct vkv_arena {
  int device = 0;
  uint64_t handle_bytes = 0;
  int32_t num_handles = 0;
  char* base = nullptr;
  std::vector<hipMemGenericAllocationHandle_t> phys;
  std::vector<uint8_t> mapped;
  hipMemAllocationProp prop{};
  hipMemAccessDesc access{};
};

namespace vkv {

static int map_one(vkv_arena* a, int32_t h) {
  hipError_t e = hipMemCreate(&a->phys[h], a->handle_bytes, &a->prop, 0);
  if (e == hipErrorOutOfMemory) {
    set_error("arena: the device has no memory left for handle %d", h);
    return VKV_E_NOSPACE;
  }
  if (e != hipSuccess) return hip_fail(e, "hipMemCreate");
  char* at = a->base + (uint64_t)h * a->handle_bytes;
  e = hipMemMap(at, a->handle_bytes, 0, a->phys[h], 0);
  if (e == hipSuccess) e = hipMemSetAccess(at, a->handle_bytes, &a->access, 1);
  if (e != hipSuccess) {
    (void)hipMemUnmap(at, a->handle_bytes);
    (void)hipMemRelease(a->phys[h]);
    return hip_fail(e, "hipMemMap / hipMemSetAccess");
  }
  a->mapped[h] = 1;
  return VKV_OK;
}

static int unmap_one(vkv_arena* a, int32_t h) {
  VKV_HIP(hipMemUnmap(a->base + (uint64_t)h * a->handle_bytes, a->handle_bytes));
  a->mapped[h] = 0;
  VKV_HIP(hipMemRelease(a->phys[h]));
  return VKV_OK;
}

bool arena_range_mapped(const vkv_arena* a, int32_t first, int32_t last) {
  for (int32_t h = first; h < last; ++h)
    if (!a->mapped[h]) return false;
  return true;
}

// the arena backs exactly this pool, and [lo, hi) lies inside one of its handed-over ranges whose tables are clean
static int check_pair(const vkv_arena* a, const vkv_pool* p, int32_t lo, int32_t hi, const char* who) {
  if (!a || !p) { set_error("%s: null arena or pool", who); return VKV_E_INVAL; }
  if (p->arena != a || (char*)p->cfg.base != a->base ||
      (uint64_t)p->cfg.blocks_per_handle * p->block_bytes != a->handle_bytes ||
      (uint64_t)p->cfg.num_blocks * p->block_bytes != (uint64_t)a->num_handles * a->handle_bytes) {
    set_error("%s: the arena is not attached to this pool (kv_pool_attach_arena)", who);
    return VKV_E_INVAL;
  }
  const int32_t bph = p->cfg.blocks_per_handle;
  if (lo < 0 || hi > p->cfg.num_blocks || lo >= hi || lo % bph || hi % bph) {
    set_error("%s: [%d,%d) must be non-empty, inside the pool and a multiple of %d blocks", who, lo, hi, bph);
    return VKV_E_INVAL;
  }
  for (const auto& r : p->released)
    if (r.first <= lo && hi <= r.second) {
      if (!r.clean) {
        set_error("%s: [%d,%d) was handed over without the device block tables being rewritten; slices may still "
                  "read it", who, lo, hi);
        return VKV_E_STATE;
      }
      return VKV_OK;
    }
  set_error("%s: [%d,%d) does not lie inside a handed-over range of the pool", who, lo, hi);
  return VKV_E_STATE;
}

}  // namespace vkv

using namespace vkv;

extern "C" {

int kv_arena_create(int32_t device, uint64_t handle_bytes, int32_t num_handles, vkv_arena** out, void** base_out) {
  if (!out || !base_out || num_handles < 1 || handle_bytes == 0) { set_error("kv_arena_create: bad argument"); return VKV_E_INVAL; }
  *out = nullptr;
  *base_out = nullptr;
  int count = 0;
  VKV_HIP(hipGetDeviceCount(&count));
  if (device < 0 || device >= count) { set_error("kv_arena_create: no device %d", device); return VKV_E_INVAL; }
  int supported = 0;
  VKV_HIP(hipDeviceGetAttribute(&supported, hipDeviceAttributeVirtualMemoryManagementSupported, device));
  if (!supported) { set_error("kv_arena_create: device %d has no virtual memory management", device); return VKV_E_INVAL; }
  vkv_arena* a = new vkv_arena;
  a->device = device;
  a->prop.type = hipMemAllocationTypePinned;
  a->prop.location.type = hipMemLocationTypeDevice;
  a->prop.location.id = device;
  a->access.location = a->prop.location;
  a->access.flags = hipMemAccessFlagsProtReadWrite;
  size_t gran = 0;
  hipError_t e = hipMemGetAllocationGranularity(&gran, &a->prop, hipMemAllocationGranularityMinimum);
  if (e != hipSuccess) { delete a; return hip_fail(e, "hipMemGetAllocationGranularity"); }
  if (gran == 0 || handle_bytes % gran) {
    set_error("kv_arena_create: handle_bytes must be a multiple of the allocation granularity (%zu)", gran);
    delete a;
    return VKV_E_INVAL;
  }
  a->handle_bytes = handle_bytes;
  a->num_handles = num_handles;
  a->phys.resize(num_handles);
  a->mapped.assign(num_handles, 0);
  void* base = nullptr;
  e = hipMemAddressReserve(&base, handle_bytes * (uint64_t)num_handles, 0, nullptr, 0);
  if (e != hipSuccess) { delete a; return hip_fail(e, "hipMemAddressReserve"); }
  a->base = (char*)base;
  for (int32_t h = 0; h < num_handles; ++h) {
    int st = map_one(a, h);
    if (st != VKV_OK) {
      for (int32_t g = 0; g < h; ++g) (void)unmap_one(a, g);
      (void)hipMemAddressFree(a->base, handle_bytes * (uint64_t)num_handles);
      delete a;
      return st;
    }
  }
  *out = a;
  *base_out = base;
  return VKV_OK;
}

int kv_arena_destroy(vkv_arena* a) {
  if (!a) return VKV_OK;
  for (int32_t h = 0; h < a->num_handles; ++h)
    if (a->mapped[h]) (void)unmap_one(a, h);
  (void)hipMemAddressFree(a->base, a->handle_bytes * (uint64_t)a->num_handles);
  delete a;
  return VKV_OK;
}

int kv_pool_attach_arena(vkv_pool* p, vkv_arena* a) {
  if (!p) { set_error("kv_pool_attach_arena: null pool"); return VKV_E_INVAL; }
  if (a && ((char*)p->cfg.base != a->base || (uint64_t)p->cfg.blocks_per_handle * p->block_bytes != a->handle_bytes ||
            (uint64_t)p->cfg.num_blocks * p->block_bytes != (uint64_t)a->num_handles * a->handle_bytes)) {
    set_error("kv_pool_attach_arena: the pool's base, handle size or size differs from the arena's");
    return VKV_E_INVAL;
  }
  p->arena = a;
  return VKV_OK;
}

int kv_arena_release(vkv_arena* a, vkv_pool* p, int32_t lo, int32_t hi) {
  int st = check_pair(a, p, lo, hi, "kv_arena_release");
  if (st != VKV_OK) return st;
  const int32_t bph = p->cfg.blocks_per_handle;
  for (int32_t h = lo / bph; h < hi / bph; ++h)
    if (!a->mapped[h]) { set_error("kv_arena_release: handle %d is not mapped", h); return VKV_E_STATE; }
  for (int32_t h = lo / bph; h < hi / bph; ++h)
    if ((st = unmap_one(a, h)) != VKV_OK) { p->broken = true; return st; }
  return VKV_OK;
}

int kv_arena_restore(vkv_arena* a, vkv_pool* p, int32_t lo, int32_t hi) {
  int st = check_pair(a, p, lo, hi, "kv_arena_restore");
  if (st != VKV_OK) return st;
  const int32_t bph = p->cfg.blocks_per_handle;
  for (int32_t h = lo / bph; h < hi / bph; ++h)
    if (a->mapped[h]) { set_error("kv_arena_restore: handle %d is mapped", h); return VKV_E_STATE; }
  for (int32_t h = lo / bph; h < hi / bph; ++h) {
    if ((st = map_one(a, h)) != VKV_OK) {
      // leave the range as it was: all of it unmapped
      for (int32_t g = lo / bph; g < h; ++g) (void)unmap_one(a, g);
      return st;
    }
  }
  return VKV_OK;
}

int kv_arena_state(vkv_arena* a, uint8_t* mapped_out, uint64_t* mapped_bytes) {
  if (!a) { set_error("kv_arena_state: null arena"); return VKV_E_INVAL; }
  uint64_t n = 0;
  for (int32_t h = 0; h < a->num_handles; ++h) {
    if (mapped_out) mapped_out[h] = a->mapped[h];
    n += a->mapped[h];
  }
  if (mapped_bytes) *mapped_bytes = n * a->handle_bytes;
  return VKV_OK;
}

}  // extern "C"
