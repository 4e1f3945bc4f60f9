// Bandwidth probes: what the memory system gives the two simplest access patterns, a
// read-only sequential stream and a plain device-to-device copy.  They are yardsticks for the
// attention and relocation kernels (both bound by HBM bandwidth), not part of the method.
#include "vkv_internal.h"

namespace vkv {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kProbeVecsPerWg = 4096;   // 64 KiB per workgroup, 16 bytes per lane and load
constexpr int kProbeUnroll = 8;         // loads in flight per lane

// Every workgroup streams one contiguous 64 KiB piece; the xor of all values is stored only if
// it equals a value the caller cannot have produced on purpose, which keeps the loads alive.
__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4* __restrict__ src, uint64_t n_vecs,
                                                         u32x4* __restrict__ sink) {
  // each wave streams a contiguous quarter of the piece (requests of a wave follow each other in address)
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint64_t first = (uint64_t)blockIdx.x * kProbeVecsPerWg + wave * (kProbeVecsPerWg / 4);
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (uint32_t i = lane; i < (uint32_t)kProbeVecsPerWg / 4; i += 64 * kProbeUnroll) {
    u32x4 r[kProbeUnroll];
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) {
      const uint64_t idx = first + i + (uint64_t)u * 64;
      r[u] = idx < n_vecs ? __builtin_nontemporal_load(src + idx) : u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int u = 0; u < kProbeUnroll; ++u) acc ^= r[u];
  }
  if (acc.x == 0x9E3779B9u && acc.y == 0x7F4A7C15u && acc.z == 0xF39CC060u && acc.w == 0x5CEDC834u)
    sink[threadIdx.x & 15] = acc;
}

}  // namespace vkv

using namespace vkv;

extern "C" {

int kv_probe_read(const void* src, uint64_t bytes, void* sink, void* stream) {
  if (!src || !sink || bytes == 0 || bytes % 16 || (uintptr_t)src % 16 || (uintptr_t)sink % 16) {
    set_error("kv_probe_read: src and sink must be 16-byte aligned device pointers, bytes a positive multiple of 16");
    return VKV_E_INVAL;
  }
  const uint64_t n_vecs = bytes / 16, wgs = (n_vecs + kProbeVecsPerWg - 1) / kProbeVecsPerWg;
  if (wgs > 0x7FFFFFFFull) { set_error("kv_probe_read: at most 128 TiB per call"); return VKV_E_INVAL; }
  hipLaunchKernelGGL(probe_read_kernel, dim3((unsigned)wgs), dim3(256), 0, (hipStream_t)stream, (const u32x4*)src,
                     n_vecs, (u32x4*)sink);
  VKV_HIP(hipGetLastError());
  return VKV_OK;
}

int kv_probe_copy(void* dst, const void* src, uint64_t bytes, void* stream) {
  if (!dst || !src || bytes == 0) { set_error("kv_probe_copy: bad argument"); return VKV_E_INVAL; }
  VKV_HIP(hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, (hipStream_t)stream));
  return VKV_OK;
}

}  // extern "C"
