// ft_submit_static: the submit for callers that cannot allocate (code under HIP graph capture,
// tight serving loops, harnesses that forbid hipMalloc). It does what ft_submit_transfers does for
// a job of pinned-host and pool sides - same validation, same chunk order, same copy kernel - but
// takes nothing from the runtime: no device buffer, no pinned buffer, no event, no stream. What the
// kernels need beyond the caller's memory (the schedule tables and the ticket counter of each link
// class) lies in one fixed array in device memory that belongs to this library, and everything is
// launched on the caller's stream.
#include <hip/hip_runtime.h>

#include <mutex>
#include <string>
#include <unordered_map>
#include <vector>

#include "ft_guard.h"
#include "ft_internal.h"

namespace ft {

// Per link class: one 256-byte line with the ticket counter, then the class's tables.
constexpr uint64_t kStaticTableBytes = 64 * 1024;
constexpr uint64_t kStaticClassBytes = 256 + kStaticTableBytes;
constexpr uint64_t kScratchBytes = FT_NCLASS * kStaticClassBytes;  // 197 376 bytes per GPU, held until the process ends

// In host code this name is a stand-in for the device array, not its address: host code uses the
// pointer that hipGetSymbolAddress returns for the current device (static_scratch below).
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kScratchBytes];

struct StaticDevice {
  unsigned char *ptr = nullptr;  // this device's copy of `scratch`
  int cu_count = 0;
};

// The scratch array of device `device`, which must be current. Looked up once per device: every
// GPU holds its own copy of the array at its own address.
int static_scratch(ft_pool *p, int device, StaticDevice *out) {
  static std::mutex mu;
  static std::unordered_map<int, StaticDevice> table;
  std::lock_guard<std::mutex> lock(mu);
  auto it = table.find(device);
  if (it != table.end()) {
    *out = it->second;
    return FT_OK;
  }
  StaticDevice sd;
  FT_HIP(p, hipGetSymbolAddress(reinterpret_cast<void **>(&sd.ptr), HIP_SYMBOL(scratch)));
  FT_HIP(p, hipDeviceGetAttribute(&sd.cu_count, hipDeviceAttributeMultiprocessorCount, device));
  if (sd.ptr == nullptr || sd.cu_count <= 0) {
    p->hip_error = "ft_submit_static: no scratch array on this device";
    return FT_EHIP;
  }
  table[device] = sd;
  *out = sd;
  return FT_OK;
}

// Writes `nwords` 8-byte words that came with the launch to dst, and (zero != null) sets the
// class's counter line back to zero: the array keeps what the last call left in it.
__global__ __launch_bounds__(kInlineBytes / 8) void ft_scratch_put_kernel(uint64_t *dst, InlineBlob blob, uint32_t nwords,
                                                                          unsigned long long *zero) {
  const uint32_t i = threadIdx.x;
  if (i < nwords) dst[i] = blob.w[i];
  if (zero != nullptr && i < 2) zero[i] = 0ull;
}

struct StaticClass {
  bool used = false;
  Layout lay;
  std::vector<Skip> skips;
  uint64_t ntickets = 0, tile_bytes = 0;
  uint32_t tiles_per_chunk = 0;
};

}  // namespace ft

using namespace ft;

extern "C" int ft_submit_static(ft_pool *p, const ft_desc *descs, uint32_t ndesc, const uint32_t *weights,
                                uint32_t nfunc, uint64_t chunk_bytes, uint32_t flags, void *hip_stream) try {
  if (p == nullptr) return FT_EINVAL;
  if (flags & ~(uint32_t)FT_VALIDATE) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  SubmitPlan plan;
  int rc = plan_submit(p->slabs, p->windows, descs, ndesc, weights, nfunc, chunk_bytes, flags, &plan);
  if (rc != FT_OK) return rc;
  if (plan.has_pageable) return FT_EINVAL;  // pageable memory needs a pinned buffer, which would be an allocation
  const bool with_p2p = plan.cls[FT_P2P].nchunks > 0;
  StaticClass sc[FT_NCLASS];
  bool any = false;
  // every class is shaped and measured before anything is launched: all or nothing
  for (int c = 0; c < FT_NCLASS; ++c) {
    ClassPlan &cp = plan.cls[c];
    if (cp.nchunks == 0) continue;
    StaticClass &s = sc[c];
    s.used = any = true;
    tile_shape(chunk_bytes, default_tile(c, with_p2p, mostly_short_rows(cp), cp.payload), &s.tile_bytes, &s.tiles_per_chunk);
    build_chunk_table(cp, chunk_bytes, s.tile_bytes, s.tiles_per_chunk);
    build_skips(cp, chunk_bytes, s.tile_bytes, s.tiles_per_chunk, &s.skips, &s.ntickets);
    s.lay = layout_of(cp, 0, 1);
    if (s.lay.end > kStaticClassBytes && cp.desc_per == 1) {
      // without the table of descriptors per chunk the decode searches the function's descriptors
      cp.chunk_desc.clear();
      s.lay = layout_of(cp, 0, 1);
    }
    if (s.lay.end > kStaticClassBytes) return FT_E2BIG;
  }
  if (!any) return FT_OK;
  DeviceGuard guard(p->device);
  StaticDevice sd;
  rc = static_scratch(p, p->device, &sd);
  if (rc != FT_OK) return rc;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  std::vector<char> h;
  InlineBlob piece;
  for (int c = 0; c < FT_NCLASS; ++c) {
    const StaticClass &s = sc[c];
    if (!s.used) continue;
    const ClassPlan &cp = plan.cls[c];
    char *d = reinterpret_cast<char *>(sd.ptr) + (uint64_t)c * kStaticClassBytes;
    h.assign(s.lay.end, 0);
    ClassTable T{};
    fill_class_table(cp, s.lay, h.data(), d, s.skips, s.ntickets, chunk_bytes, s.tile_bytes, s.tiles_per_chunk, &T);
    // the tables reach the array in pieces that travel with small launches; the first one also
    // clears the counter. On one stream these launches and the copy kernel run one after another.
    const uint64_t first = s.lay.phases, last = s.lay.end;  // the counter line is not uploaded
    bool zeroed = false;
    for (uint64_t at = first; at < last || !zeroed; at += kInlineBytes) {
      const uint64_t n = at < last ? (last - at < kInlineBytes ? last - at : kInlineBytes) : 0;
      std::memcpy(piece.w, h.data() + at, n);
      hipLaunchKernelGGL(ft_scratch_put_kernel, dim3(1), dim3(kInlineBytes / 8), 0, stream,
                         reinterpret_cast<uint64_t *>(d + at), piece, (uint32_t)((n + 7) / 8),
                         zeroed ? nullptr : T.ticket);
      FT_HIP(p, hipGetLastError());
      zeroed = true;
    }
    uint64_t wg = c == FT_P2P ? (uint64_t)sd.cu_count : (with_p2p || c == FT_P2H) ? 32u : 64u;
    if (wg > T.ntickets) wg = T.ntickets;
    FT_HIP(p, launch_copy(T, c, (uint32_t)wg, stream, nullptr, nullptr));
  }
  return FT_OK;
}
FT_CATCH_ALL
