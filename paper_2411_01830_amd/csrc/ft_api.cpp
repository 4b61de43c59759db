// C ABI of the transfer engine: pool handle, jobs, streams, table upload, launches.
#include <hip/hip_runtime_api.h>

#include <chrono>
#include <cmath>
#include <cstring>
#include <memory>
#include <mutex>
#include <string>
#include <unordered_map>
#include <vector>

#include "ft_internal.h"
#include "ft_guard.h"

namespace ft {

DeviceCtx *device_ctx(int device) {
  static std::mutex table_mu;
  static std::unordered_map<int, DeviceCtx *> table;
  std::lock_guard<std::mutex> lock(table_mu);
  auto it = table.find(device);
  if (it != table.end()) return it->second;
  DeviceCtx *c = new DeviceCtx();  // never freed: must outlive every pool and static destructors
  c->device = device;
  table[device] = c;
  return c;
}

int ensure_device(ft_pool *p) {
  DeviceCtx *c = p->ctx;
  std::lock_guard<std::mutex> lock(c->mu);
  if (c->ready) return FT_OK;
  int count = 0;
  FT_HIP(p, hipGetDeviceCount(&count));
  if (p->device < 0 || p->device >= count) {
    p->hip_error = "device ordinal out of range";
    return FT_EHIP;
  }
  FT_HIP(p, hipDeviceGetAttribute(&c->cu_count, hipDeviceAttributeMultiprocessorCount, p->device));
  FT_HIP(p, hipDeviceGetAttribute(&c->clock_khz, hipDeviceAttributeWallClockRate, p->device));
  for (int k = 0; k < FT_NCLASS; ++k)
    if (c->streams[k] == nullptr) FT_HIP(p, hipStreamCreateWithFlags(&c->streams[k], hipStreamNonBlocking));
  for (int k = 0; k < FT_NCLASS; ++k)
    if (c->alt_streams[k] == nullptr) FT_HIP(p, hipStreamCreateWithFlags(&c->alt_streams[k], hipStreamNonBlocking));
  if (c->idle_counter == nullptr) {
    constexpr uint32_t kPairs = 256;
    FT_HIP(p, hipMalloc(reinterpret_cast<void **>(&c->idle_counter), 256 + kPairs * 16));
    FT_HIP(p, hipMemset(c->idle_counter, 0, 256 + kPairs * 16));
    c->counter_pairs = c->idle_counter + 256 / sizeof(unsigned long long);
    for (uint32_t i = 0; i < kPairs; ++i) c->free_pairs.push_back(kPairs - 1 - i);
  }
  c->ready = true;
  return FT_OK;
}

uint64_t round_pow2(uint64_t v, uint64_t floor_) {
  uint64_t c = floor_;
  while (c < v) c <<= 1;
  return c;
}

int get_blob(ft_pool *p, uint64_t need, bool pinned_twin, Blob *out) {
  std::lock_guard<std::mutex> lock(p->ctx->mu);
  std::vector<Blob> &cache = pinned_twin ? p->ctx->free_blobs : p->ctx->free_dev_blobs;
  size_t best = cache.size();
  for (size_t i = 0; i < cache.size(); ++i)
    if (cache[i].cap >= need && (best == cache.size() || cache[i].cap < cache[best].cap)) best = i;
  if (best != cache.size()) {
    *out = cache[best];
    cache.erase(cache.begin() + (long)best);
    return FT_OK;
  }
  Blob b;
  b.cap = round_pow2(need, 64 * 1024);
  FT_HIP(p, hipMalloc(reinterpret_cast<void **>(&b.dev), b.cap));
  if (pinned_twin) {
    hipError_t e = hipHostMalloc(reinterpret_cast<void **>(&b.host), b.cap, hipHostMallocDefault);
    if (e != hipSuccess) {
      (void)hipFree(b.dev);
      p->hip_error = std::string("hipHostMalloc: ") + hipGetErrorString(e);
      return FT_EHIP;
    }
  }
  *out = b;
  return FT_OK;
}

void put_blob(ft_pool *p, Blob &b) {
  if (b.dev == nullptr) return;
  std::lock_guard<std::mutex> lock(p->ctx->mu);
  (b.host ? p->ctx->free_blobs : p->ctx->free_dev_blobs).push_back(b);
  b = Blob();
}

int get_event(ft_pool *p, bool timing, hipEvent_t *out) {
  std::lock_guard<std::mutex> lock(p->ctx->mu);
  std::vector<hipEvent_t> &cache = timing ? p->ctx->free_timing_events : p->ctx->free_events;
  if (!cache.empty()) {
    *out = cache.back();
    cache.pop_back();
    return FT_OK;
  }
  FT_HIP(p, hipEventCreateWithFlags(out, timing ? hipEventDefault : hipEventDisableTiming));
  return FT_OK;
}

void put_event(ft_pool *p, bool timing, hipEvent_t &e) {
  if (e == nullptr) return;
  std::lock_guard<std::mutex> lock(p->ctx->mu);
  (timing ? p->ctx->free_timing_events : p->ctx->free_events).push_back(e);
  e = nullptr;
}

uint64_t align_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

int get_pinned(ft_pool *p, uint64_t need, char **out, uint64_t *cap) {
  {
    std::lock_guard<std::mutex> lock(p->ctx->mu);
    auto &cache = p->ctx->free_pinned;
    size_t best = cache.size();
    for (size_t i = 0; i < cache.size(); ++i)
      if (cache[i].second >= need && (best == cache.size() || cache[i].second < cache[best].second)) best = i;
    if (best != cache.size()) {
      *out = cache[best].first;
      *cap = cache[best].second;
      cache.erase(cache.begin() + (long)best);
      return FT_OK;
    }
  }
  const uint64_t bytes = round_pow2(need, 1 << 20);
  FT_HIP(p, hipHostMalloc(reinterpret_cast<void **>(out), bytes, hipHostMallocDefault));
  *cap = bytes;
  return FT_OK;
}

void put_pinned(ft_pool *p, char *ptr, uint64_t cap) {
  if (ptr == nullptr) return;
  std::lock_guard<std::mutex> lock(p->ctx->mu);
  p->ctx->free_pinned.push_back({ptr, cap});
}

Layout layout_of(const ClassPlan &cp, uint64_t base, uint64_t ncounters) {
  Layout l;
  l.ticket = align_up(base, 256);
  // the counters of successive launches sit 8 bytes apart: one launch runs at a time
  l.phases = l.ticket + align_up(ncounters * 8, 256);
  l.slots = align_up(l.phases + cp.phases.size() * sizeof(Phase), 64);
  l.funcs = align_up(l.slots + cp.slots.size() * sizeof(Slot), 64);
  l.xfers = align_up(l.funcs + cp.funcs.size() * sizeof(Func), 64);
  l.chunks = align_up(l.xfers + cp.xfers.size() * sizeof(Xfer), 64);
  l.skips = align_up(l.chunks + cp.chunk_desc.size() * sizeof(uint32_t), 64);
  // at most one run of empty tiles per function
  l.end = align_up(l.skips + cp.funcs.size() * sizeof(Skip), 256);
  return l;
}

Layout inline_layout_of(const ClassPlan &cp) {
  Layout l;
  l.ticket = 0;
  l.phases = 0;
  l.slots = align_up(l.phases + cp.phases.size() * sizeof(Phase), 16);
  l.funcs = align_up(l.slots + cp.slots.size() * sizeof(Slot), 16);
  l.xfers = align_up(l.funcs + cp.funcs.size() * sizeof(Func), 16);
  l.chunks = align_up(l.xfers + cp.xfers.size() * sizeof(Xfer), 16);
  l.skips = align_up(l.chunks + cp.chunk_desc.size() * sizeof(uint32_t), 16);
  l.end = l.skips + cp.funcs.size() * sizeof(Skip);
  return l;
}

void fill_tables(const ClassPlan &cp, const Layout &lay, char *h, char *d, ClassTable *T) {
  copy_table(h + lay.phases, cp.phases);
  copy_table(h + lay.slots, cp.slots);
  copy_table(h + lay.funcs, cp.funcs);
  copy_table(h + lay.xfers, cp.xfers);
  copy_table(h + lay.chunks, cp.chunk_desc);
  const uintptr_t base = reinterpret_cast<uintptr_t>(d);
  T->phases = reinterpret_cast<const Phase *>(base + lay.phases);
  T->slots = reinterpret_cast<const Slot *>(base + lay.slots);
  T->funcs = reinterpret_cast<const Func *>(base + lay.funcs);
  T->xfers = reinterpret_cast<const Xfer *>(base + lay.xfers);
  T->chunk_desc = cp.chunk_desc.empty() ? nullptr : reinterpret_cast<const uint32_t *>(base + lay.chunks);
  T->skips = reinterpret_cast<const Skip *>(base + lay.skips);
  T->ticket = d == nullptr ? nullptr : reinterpret_cast<unsigned long long *>(base + lay.ticket);
  T->log = nullptr;
  T->wg_log = nullptr;
  T->nchunks = cp.nchunks;
  T->nphases = (uint32_t)cp.phases.size();
  T->nfuncs = (uint32_t)cp.funcs.size();
  T->desc_per = cp.desc_per;
  T->inline_tables = d == nullptr ? 1u : 0u;
  T->self_reset = 0;
  T->single = 0;
  T->stage_base = 0;
  T->stage_rank0 = 0;
  T->stage_slot0 = 0;
  T->ticket_base = 0;
  T->skip_acc0 = 0;
  T->skip0 = 0;
  T->phase0 = 0;
  T->first_phase = Phase{};
  T->first_next_base = ~0ull;
  T->first_skip_at = ~0ull;
}

bool mostly_short_rows(const ClassPlan &cp) {
  uint64_t short_bytes = 0;
  for (const Xfer &x : cp.xfers)
    if (x.rows > 1 && x.row_bytes <= 2048) short_bytes += x.row_bytes * x.rows;
  return 2 * short_bytes > cp.payload;
}

// Launch shape when the caller has not tuned it.
//
// pool->pool is bound by HBM. One workgroup per CU, each holding a whole 64 KiB tile in
// registers, keeps the addresses in flight inside a window of a few MiB, which the
// memory controllers serve best; more resident workgroups measured slower.
//
// The host link needs little in flight: about 256 KiB of outstanding reads already
// reach 96 % of what the copy engines get, 1 MiB reaches all of it. Every outstanding
// host access holds a slot on the path from L2 to the fabric for microseconds, and
// pool->pool traffic queues behind it: with 4 MiB of host reads in flight a concurrent
// pool->pool kernel ran 20x slower. So a job that carries both kinds keeps 256 KiB of
// host accesses in flight per class; a job with host traffic only uses 64 x 16 KiB for
// host->pool. pool->host, whose stores are written through to the link as they are issued: 64 x
// 16 KiB for jobs without pool->pool traffic (one 16 MiB tensor 305 us and one of 64 MiB 1187 us,
// within 1 % of the runtime's copy, against 315 and 1249 us at 32 x 8 KiB; the tiny workload's 32
// tensors 96 % against 95 % of the link), 8 KiB tiles up to 256 KiB of payload (64 KiB: 12.3 against
// 12.7 us), and 32 x 8 KiB beside pool->pool traffic, whose workgroups a host-link workgroup on the
// same compute unit slows down.
// Host->pool beside pool->pool traffic: 16 workgroups of 16 KiB keep the link as full as 32 of 8 KiB do
// (256 KiB of reads in flight either way) and slow half as many compute units' pool->pool workgroups
// (large_mixed: link 56.7 -> 57.0 GB/s, pool->pool launches 82.6 -> 81.8 us).
uint32_t default_workgroups(const ft_pool *p, int cls, bool with_p2p) {
  if (cls == FT_P2P) return (uint32_t)p->ctx->cu_count;
  if (cls == FT_P2H) return with_p2p ? 32u : 64u;
  return with_p2p ? 16u : 64u;
}

// short_rows: most of the class's payload sits in pitched descriptors with rows of at
// most 2 KiB (a gather of image crops). Such a job is bound by latency and by what a compute
// unit's memory pipeline does with windows of 16 bytes at any address, not by HBM: it runs the
// kernel's light build (blocks of 16 KiB instead of 64 KiB, under 200 registers per lane), two
// workgroups per compute unit, and a tile costs a few microseconds whatever its size (its
// ticket - the counter hands out about 70 million a second, all workgroups together -, the
// decode, the barriers, a memory round trip per piece). Crops of the traffic workload, 512
// workgroups: 47.7 us at 16 KiB tiles, 39.8 at 26 KiB, 38.1 at 43 KiB, 39.1 at 64 KiB (fewer
// than two tiles per workgroup are left to balance the launch's end).
uint64_t default_tile(int cls, bool with_p2p, bool short_rows, uint64_t payload) {
  if (cls == FT_P2P) return short_rows ? 43u * 1024u : 64u * 1024u;
  if (cls == FT_P2H) return with_p2p || payload <= 256u * 1024u ? 8u * 1024u : 16u * 1024u;
  return 16u * 1024u;
}

hipMemcpyKind kind_of(int cls) {
  return cls == FT_H2P ? hipMemcpyHostToDevice : cls == FT_P2H ? hipMemcpyDeviceToHost : hipMemcpyDeviceToDevice;
}

// The comparison path: the same chunk order, one copy-engine call per chunk piece.
int run_dma(ft_pool *p, const ClassPlan &cp, uint64_t C, int cls, hipStream_t stream) {
  const hipMemcpyKind kind = kind_of(cls);
  for (uint64_t rank = 0; rank < cp.nchunks; ++rank) {
    const ChunkId id = decode_rank(cp.phases.data(), (uint32_t)cp.phases.size(), cp.slots.data(), rank);
    const Func &fn = cp.funcs[id.fl];
    uint64_t pos = (fn.chunk_base + id.k) * C;
    uint64_t end = pos + C < fn.stream_bytes ? pos + C : fn.stream_bytes;
    uint32_t x = find_xfer(cp.xfers.data(), fn.desc_off, fn.desc_off + fn.ndesc - 1, pos);
    while (pos < end) {
      const Xfer &X = cp.xfers[x];
      uint64_t q = pos - X.stream_off;
      uint64_t take = X.row_bytes * X.rows - q;
      if (take > end - pos) take = end - pos;
      if (X.rows == 1) {
        FT_HIP(p, hipMemcpyAsync(reinterpret_cast<void *>(X.dst + q), reinterpret_cast<void *>(X.src + q),
                                 take, kind, stream));
      } else {
        uint64_t r = q / X.row_bytes, c = q % X.row_bytes, left = take;
        if (c != 0) {  // rest of a row that was begun by the previous chunk
          uint64_t n = X.row_bytes - c < left ? X.row_bytes - c : left;
          FT_HIP(p, hipMemcpyAsync(reinterpret_cast<void *>(X.dst + r * X.dst_pitch + c),
                                   reinterpret_cast<void *>(X.src + r * X.src_pitch + c), n, kind, stream));
          left -= n;
          r += 1;
        }
        uint64_t full = left / X.row_bytes;
        if (full > 0) {
          FT_HIP(p, hipMemcpy2DAsync(reinterpret_cast<void *>(X.dst + r * X.dst_pitch), X.dst_pitch,
                                     reinterpret_cast<void *>(X.src + r * X.src_pitch), X.src_pitch,
                                     X.row_bytes, full, kind, stream));
          left -= full * X.row_bytes;
          r += full;
        }
        if (left > 0)
          FT_HIP(p, hipMemcpyAsync(reinterpret_cast<void *>(X.dst + r * X.dst_pitch),
                                   reinterpret_cast<void *>(X.src + r * X.src_pitch), left, kind, stream));
      }
      pos += take;
      ++x;
    }
  }
  return FT_OK;
}

void retire(ft_pool *p, Job *job) {
  for (size_t i = 0; i < job->allocs.size(); ++i) {
    Allocation *al = p->slabs.at(job->allocs[i]);
    // (the allocation may have been returned in stream order meanwhile and its offset handed out again)
    if (al && al->serial == job->alloc_serials[i] && al->busy > 0) al->busy -= 1;
  }
  job->allocs.clear();
  job->alloc_serials.clear();
}

// The allocations a job refers to stay busy until it has been waited for.
void hold_allocations(ft_pool *p, Job *job, const std::vector<uint64_t> &allocs) {
  job->allocs = allocs;
  job->alloc_serials.assign(allocs.size(), 0);
  for (size_t i = 0; i < allocs.size(); ++i) {
    Allocation *al = p->slabs.at(allocs[i]);
    if (al) {
      al->busy += 1;
      job->alloc_serials[i] = al->serial;
    }
  }
}

uint32_t slab_busy(ft_pool *p, uint64_t off) {
  std::lock_guard<std::mutex> lock(p->mu);
  Allocation *al = p->slabs.at(off);
  return al ? al->busy : 0;
}

int slab_free_ordered(ft_pool *p, uint64_t off) {
  std::lock_guard<std::mutex> lock(p->mu);
  return p->slabs.free(off, true);
}

void release_device_side(ft_pool *p, Job *job) {
  put_blob(p, job->tables);
  put_pinned(p, job->bounce, job->bounce_cap);
  job->bounce = nullptr;
  job->unstage.clear();
  for (int c = 0; c < FT_NCLASS; ++c) {
    if (job->run[c].counter_pair >= 0) {
      // the kernel is over (the job was waited for, or its launch failed and the device was
      // drained), so the pair is back at zero
      std::lock_guard<std::mutex> lock(p->ctx->mu);
      p->ctx->free_pairs.push_back((uint32_t)job->run[c].counter_pair);
      job->run[c].counter_pair = -1;
    }
    put_blob(p, job->run[c].log);
    put_event(p, true, job->run[c].ev_begin);
    put_event(p, true, job->run[c].ev_end);
    put_event(p, false, job->run[c].ev_done);
  }
}

int wait_locked(ft_pool *p, Job *job) {
  DeviceGuard guard(p->device);
  for (int c = 0; c < FT_NCLASS; ++c) {
    ClassRun &r = job->run[c];
    if (!r.used) continue;
    FT_HIP(p, hipEventSynchronize(r.ev_done));
    if (job->flags & FT_TIMING) {
      FT_HIP(p, hipEventElapsedTime(&r.device_ms, r.ev_begin, r.ev_end));
      hipEvent_t epoch = nullptr;
      {
        std::lock_guard<std::mutex> ctx_lock(p->ctx->mu);
        epoch = p->ctx->epoch;
      }
      // an epoch recorded after the job began gives no usable time: leave -1
      if (epoch != nullptr && hipEventElapsedTime(&r.begin_ms, epoch, r.ev_begin) == hipSuccess &&
          hipEventElapsedTime(&r.end_ms, epoch, r.ev_end) == hipSuccess) {
      } else {
        (void)hipGetLastError();
        r.begin_ms = r.end_ms = -1.f;
      }
    }
    if ((job->flags & FT_LOG) && r.log.dev != nullptr) {
      r.log_host.resize(r.table.ntickets);
      FT_HIP(p, hipMemcpy(r.log_host.data(), r.log.dev, r.table.ntickets * sizeof(LogEntry),
                          hipMemcpyDeviceToHost));
      r.wg_log_host.resize(r.workgroups);
      FT_HIP(p, hipMemcpy(r.wg_log_host.data(), r.log.dev + r.table.ntickets * sizeof(LogEntry),
                          r.workgroups * sizeof(WgLogEntry), hipMemcpyDeviceToHost));
    }
  }
  job->waited = true;
  retire(p, job);
  return FT_OK;
}

}  // namespace ft

namespace ft {

// Tile shape per class, then the descriptor table and the runs of empty tiles that go with it.
void shape_classes(ft_pool *p, Job *job, SubmitPlan &plan, uint64_t chunk_bytes) {
  const bool with_p2p = plan.cls[FT_P2P].nchunks > 0;
  for (int c = 0; c < FT_NCLASS; ++c) {
    ClassPlan &cp = plan.cls[c];
    if (cp.nchunks == 0) continue;
    ClassRun &r = job->run[c];
    const Tuning &tn = p->tuning[c];
    const bool short_rows = mostly_short_rows(cp);
    r.light = c == FT_P2P && short_rows && tn.workgroups == 0;
    tile_shape(chunk_bytes, tn.tile_bytes ? tn.tile_bytes : default_tile(c, with_p2p, short_rows, cp.payload),
               &r.tile_bytes, &r.tiles_per_chunk);
    build_chunk_table(cp, chunk_bytes, r.tile_bytes, r.tiles_per_chunk);
    build_skips(cp, chunk_bytes, r.tile_bytes, r.tiles_per_chunk, &r.skips, &r.table.ntickets);
  }
}

// A submit that fails after it has taken device resources hands them back.
int fail_submit(ft_pool *p, Job *job, int code) {
  // work already queued may still read the tables: drain it before they are recycled
  if (job->tables.dev != nullptr) (void)hipDeviceSynchronize();
  release_device_side(p, job);
  return code;
}

// A closed job may name pageable host memory if that is little (kBounceBytes in all): the
// sources are copied into a pinned buffer here, before the launch, the destinations are written
// there by the device and copied on by ft_wait. The descriptors are redirected, rows packed, so
// everything after this sees an ordinary job on pinned memory - including the route on which a
// small job travels with its launch. Longer pageable traffic belongs into an open job, whose
// ring overlaps these copies with the link.
constexpr uint64_t kBounceBytes = 8ull << 20;

int stage_closed_job(ft_pool *p, Job *job, SubmitPlan &plan) {
  uint64_t total = 0;
  for (ClassPlan &cp : plan.cls)
    for (const Xfer &x : cp.xfers)
      if (x.staged) total += (x.row_bytes * x.rows + 15) / 16 * 16;
  if (total > kBounceBytes) return FT_EINVAL;
  int rc = get_pinned(p, total, &job->bounce, &job->bounce_cap);
  if (rc != FT_OK) return rc;
  uint64_t at = 0;
  std::vector<HostCopy> in;
  for (ClassPlan &cp : plan.cls)
    for (Xfer &x : cp.xfers) {
      if (!x.staged) continue;
      char *slot = job->bounce + at;
      at += (x.row_bytes * x.rows + 15) / 16 * 16;
      for (uint64_t r = 0; r < x.rows; ++r) {
        if (x.staged & kStagedSrc)
          in.push_back(HostCopy{slot + r * x.row_bytes, reinterpret_cast<const char *>(x.src + r * x.src_pitch), x.row_bytes});
        else
          job->unstage.push_back(HostCopy{reinterpret_cast<char *>(x.dst + r * x.dst_pitch), slot + r * x.row_bytes, x.row_bytes});
      }
      if (x.staged & kStagedSrc) {
        x.src = reinterpret_cast<uint64_t>(slot);
        x.src_pitch = x.row_bytes;
      } else {
        x.dst = reinterpret_cast<uint64_t>(slot);
        x.dst_pitch = x.row_bytes;
      }
      x.staged = 0;
    }
  run_host_copies(p, in);
  return FT_OK;
}

// What a closed job with pageable destinations still owes once its device work is done.
void finish_staging(ft_pool *p, Job *job) {
  if (job->unstage.empty()) return;
  run_host_copies(p, job->unstage);
  job->unstage.clear();
}

// A class's table header once its tables lie at `d` (or, d = null, travel with the launch), for the
// tile shape and the runs of empty tiles chosen for it; the tables themselves are copied to `h`.
void fill_class_table(const ClassPlan &cp, const Layout &lay, char *h, char *d, const std::vector<Skip> &skips,
                      uint64_t ntickets, uint64_t chunk_bytes, uint64_t tile_bytes, uint32_t tiles_per_chunk,
                      ClassTable *T) {
  fill_tables(cp, lay, h, d, T);
  T->ntickets = ntickets;
  copy_table(h + lay.skips, skips);
  T->nskips = (uint32_t)skips.size();
  set_cursor_start(*T, cp.phases.data(), (uint32_t)cp.phases.size(), skips.data(), T->nskips);
  T->chunk_bytes = chunk_bytes;
  T->tile_bytes = tile_bytes;
  T->tiles_per_chunk = tiles_per_chunk;
}

// What is the same for both ways of launching: the class's table header and the events of the class.
int prepare_class(ft_pool *p, Job *job, int c, const ClassPlan &cp, const Layout &lay, char *h, char *d,
                  uint64_t chunk_bytes, bool timing) {
  ClassRun &r = job->run[c];
  fill_class_table(cp, lay, h, d, r.skips, r.table.ntickets /* from shape_classes */, chunk_bytes, r.tile_bytes,
                   r.tiles_per_chunk, &r.table);
  r.used = true;
  int rc = get_event(p, false, &r.ev_done);
  if (rc == FT_OK && timing) rc = get_event(p, true, &r.ev_begin);
  if (rc == FT_OK && timing) rc = get_event(p, true, &r.ev_end);
  return rc;
}

// Largest single tensor that is copied with ordinary (cached) loads and stores: with its copy it
// still fits the chip's 256 MiB last-level cache.
constexpr uint64_t kCacheResidentBytes = 128ull << 20;

// A job of one link class whose tables fit into a kernel argument is launched on the
// caller's stream itself, tables in the launch: one launch and one event record instead
// of a table upload, a fork and a join across streams - 4 us of host time instead of
// 35 us, which is most of what passing a small tensor costs. If every ticket can have a
// workgroup of its own the counter is never consulted; a larger job takes one of the
// device's self-resetting counters (unless FT_DETACHED asks that the caller's stream be
// left alone for what may be a long time). *launched says whether the job went this way.
int launch_with_the_launch(ft_pool *p, Job *job, SubmitPlan &plan, uint64_t chunk_bytes, uint32_t flags,
                           hipStream_t user, bool *launched) {
  *launched = false;
  int only = -1;
  for (int c = 0; c < FT_NCLASS; ++c)
    if (plan.cls[c].nchunks > 0) only = only == -1 ? c : -2;
  if (only < 0 || (flags & FT_PATH_DMA) || p->tuning[only].workgroups != 0) return FT_OK;
  ClassPlan &cp = plan.cls[only];
  ClassRun &r = job->run[only];
  Layout lay = inline_layout_of(cp);
  if (lay.end > kInlineBytes && cp.desc_per == 1 && cp.xfers.size() <= 4 * cp.funcs.size()) {
    // few descriptors per function: the search over a function's descriptors is short
    // enough without the table of descriptors per chunk, which is most of the bytes
    bool few = true;
    for (const Func &f : cp.funcs) few = few && f.ndesc <= 4;
    if (few) {
      cp.chunk_desc.clear();
      lay = inline_layout_of(cp);
    }
  }
  if (lay.end > kInlineBytes) return FT_OK;
  const uint64_t ntickets = r.table.ntickets;
  // host->pool: more than 64 tiles of 16 KiB requested at once is more than the link
  // takes (2 MiB as 128 x 16 KiB: 52 us; as 64 workgroups drawing tickets: 43 us)
  const uint64_t most = only == FT_P2P ? (r.light ? 2u : 1u) * (uint64_t)p->ctx->cu_count : only == FT_H2P ? 64u : 128u;
  // one contiguous transfer between 16-byte aligned addresses (any length): the workgroups share the tiles out
  // themselves (ClassTable::single >= 2)
  const bool direct = cp.funcs.size() == 1 && cp.xfers.size() == 1 && cp.funcs[0].chunk_base == 0 && !(flags & FT_LOG) &&
                      cp.xfers[0].rows == 1 && ((cp.xfers[0].src | cp.xfers[0].dst) & 15) == 0;
  const bool each_its_own = !direct && ntickets <= most;
  // a job with more tiles than that holds the caller's stream for a while: not what FT_DETACHED asked for
  if (ntickets > most && (flags & FT_DETACHED)) return FT_OK;
  if (!each_its_own && !direct) {
    std::lock_guard<std::mutex> ctx_lock(p->ctx->mu);
    if (p->ctx->free_pairs.empty()) return FT_OK;
    r.counter_pair = (int)p->ctx->free_pairs.back();
    p->ctx->free_pairs.pop_back();
  }
  job->inline_tables.reset(new InlineBlob());
  char *h = reinterpret_cast<char *>(job->inline_tables->w);
  int rc = prepare_class(p, job, only, cp, lay, h, nullptr, chunk_bytes, (flags & FT_TIMING) != 0);
  if (rc != FT_OK) return fail_submit(p, job, rc);
  ClassTable &T = r.table;
  T.single = cp.funcs.size() == 1 && cp.xfers.size() == 1 && cp.funcs[0].chunk_base == 0 ? 1u : 0u;
  uint64_t wg = ntickets;
  if (direct) {
    T.ticket = p->ctx->idle_counter;  // never consulted
    // A tensor that fits the last-level cache together with its copy (256 MiB on this chip) moves with
    // ordinary loads and stores: its producer has just written it and its consumer is about to read the
    // copy, so both may be served from that cache (64 MiB: 26 -> 20 us, 128 MiB: 51 -> 36 us when the
    // source is still there). Larger ones stream past the caches like every other pool->pool transfer.
    T.single = only == FT_P2P && cp.payload <= kCacheResidentBytes ? 3u : 2u;
    // Host->pool: the link is full with 256 KiB of reads in flight, and a lone transfer is the faster the
    // less is asked for at once beyond that (1 MiB: 64 workgroups x 16 KiB 25 us, 16 x 16 KiB 21 us).
    wg = only == FT_H2P ? 16u : default_workgroups(p, only, only == FT_P2P);
    if (wg > ntickets) wg = ntickets;
  } else if (each_its_own) {
    T.ticket = p->ctx->idle_counter;
  } else {
    T.ticket = p->ctx->counter_pairs + 2 * r.counter_pair;
    T.self_reset = 1;
    wg = (r.light ? 2u : 1u) * default_workgroups(p, only, only == FT_P2P);
    if (wg > ntickets) wg = ntickets;
  }
  r.workgroups = (uint32_t)wg;
  r.on_user_stream = true;
  if (flags & FT_LOG) {
    rc = get_blob(p, T.ntickets * sizeof(LogEntry) + wg * sizeof(WgLogEntry), false, &r.log);
    if (rc != FT_OK) return fail_submit(p, job, rc);
    T.log = reinterpret_cast<LogEntry *>(r.log.dev);
    T.wg_log = reinterpret_cast<WgLogEntry *>(r.log.dev + T.ntickets * sizeof(LogEntry));
  }
  hipError_t e;
  if (r.ev_begin == nullptr) {
    // the done event is bound to the dispatch itself (it fires with the kernel's own completion
    // signal) instead of being a marker queued behind it: 2 us less from submit to the end of wait
    e = launch_copy(T, r.light ? kLightPoolToPool : only, r.workgroups, user, nullptr, r.ev_done, job->inline_tables.get());
  } else {
    e = launch_copy(T, r.light ? kLightPoolToPool : only, r.workgroups, user, r.ev_begin, r.ev_end, job->inline_tables.get());
    if (e == hipSuccess) e = hipEventRecord(r.ev_done, user);
  }
  if (e != hipSuccess) {
    p->hip_error = std::string("launch on the caller's stream: ") + hipGetErrorString(e);
    (void)hipDeviceSynchronize();  // the kernel may be running: its counter pair must be back at zero
    return fail_submit(p, job, FT_EHIP);
  }
  *launched = true;
  return FT_OK;
}

// The general way: the tables of all classes in one blob, copied to the device on the caller's
// stream; each class's stream waits for that copy, runs its kernel (or, FT_PATH_DMA, its chunk
// copies) and the caller's stream waits for it unless FT_DETACHED.
int launch_with_uploaded_tables(ft_pool *p, Job *job, SubmitPlan &plan, uint64_t chunk_bytes, uint32_t flags,
                                hipStream_t user) {
  const bool timing = (flags & FT_TIMING) != 0;
  const bool dma = (flags & FT_PATH_DMA) != 0;
  const bool with_p2p = plan.cls[FT_P2P].nchunks > 0;
  Layout lay[FT_NCLASS];
  uint64_t total = 0;
  for (int c = 0; c < FT_NCLASS; ++c) {
    lay[c] = layout_of(plan.cls[c], total, 1);
    if (plan.cls[c].nchunks > 0) total = lay[c].end;
  }
  int rc = get_blob(p, total, true, &job->tables);
  if (rc != FT_OK) return fail_submit(p, job, rc);
  std::memset(job->tables.host, 0, total);
  for (int c = 0; c < FT_NCLASS; ++c) {
    const ClassPlan &cp = plan.cls[c];
    if (cp.nchunks == 0) continue;
    ClassRun &r = job->run[c];
    rc = prepare_class(p, job, c, cp, lay[c], job->tables.host, job->tables.dev, chunk_bytes, timing);
    if (rc != FT_OK) return fail_submit(p, job, rc);
    ClassTable &T = r.table;
    const Tuning &tn = p->tuning[c];
    uint64_t wg = tn.workgroups ? tn.workgroups : (r.light ? 2u : 1u) * default_workgroups(p, c, with_p2p);
    if (wg > T.ntickets) wg = T.ntickets;
    r.workgroups = dma ? 0 : (uint32_t)wg;
    if ((flags & FT_LOG) && !dma) {
      rc = get_blob(p, T.ntickets * sizeof(LogEntry) + wg * sizeof(WgLogEntry), false, &r.log);
      if (rc != FT_OK) return fail_submit(p, job, rc);
      T.log = reinterpret_cast<LogEntry *>(r.log.dev);
      T.wg_log = reinterpret_cast<WgLogEntry *>(r.log.dev + T.ntickets * sizeof(LogEntry));
    }
  }

  // A job of one link class that the caller's stream is to wait for anyway runs on that stream itself:
  // table upload, kernel, done event bound to the dispatch - three runtime calls instead of seven
  // (no fork event, no wait on either side; the feature job: 57 -> 30 us inside ft_submit_transfers).
  int nused = 0;
  for (int c = 0; c < FT_NCLASS; ++c) nused += job->run[c].used ? 1 : 0;
  const bool straight = nused == 1 && !(flags & FT_DETACHED) && !dma;

  // tables (and the zeroed ticket counters) travel on the caller's stream, then fork
  hipEvent_t fork = nullptr;
  rc = get_event(p, false, &fork);
  if (rc != FT_OK) return fail_submit(p, job, rc);
  auto hip_fail = [&](hipError_t e, const char *what) {
    p->hip_error = std::string(what) + ": " + hipGetErrorString(e);
    put_event(p, false, fork);
    return fail_submit(p, job, FT_EHIP);
  };
  hipError_t e = hipMemcpyAsync(job->tables.dev, job->tables.host, total, hipMemcpyHostToDevice, user);
  if (e != hipSuccess) return hip_fail(e, "hipMemcpyAsync(tables)");
  if (!straight) {
    e = hipEventRecord(fork, user);
    if (e != hipSuccess) return hip_fail(e, "hipEventRecord(fork)");
  }
  for (int c = 0; c < FT_NCLASS; ++c) {
    ClassRun &r = job->run[c];
    if (!r.used) continue;
    if (straight) {
      r.stream = user;
      if (timing) {
        e = launch_copy(r.table, r.light ? kLightPoolToPool : c, r.workgroups, user, r.ev_begin, r.ev_end);
        if (e == hipSuccess) e = hipEventRecord(r.ev_done, user);
      } else {
        e = launch_copy(r.table, r.light ? kLightPoolToPool : c, r.workgroups, user, nullptr, r.ev_done);
      }
      if (e != hipSuccess) return hip_fail(e, "launch on the caller's stream");
      continue;
    }
    hipStream_t s = p->ctx->streams[c];
    const bool two_lanes = (flags & FT_DETACHED) && c == FT_P2P && !dma;
    if (two_lanes) {
      // only the on-device class: a host-link launch lasts milliseconds at the link's rate, so it has
      // nothing to gain, and two of them side by side would double the host reads in flight
      std::lock_guard<std::mutex> ctx_lock(p->ctx->mu);
      DeviceCtx &cx = *p->ctx;
      if (cx.lane_marker[c] == nullptr) {
        e = hipEventCreateWithFlags(&cx.lane_marker[c], hipEventDisableTiming);
        if (e != hipSuccess) return hip_fail(e, "hipEventCreateWithFlags(lane marker)");
        cx.detached_lane[c] = 1;  // nothing is running: the first launch takes the first stream
      }
      const bool last_still_runs = hipEventQuery(cx.lane_marker[c]) == hipErrorNotReady;
      const bool host_link_busy = cx.hostlink_marker != nullptr && hipEventQuery(cx.hostlink_marker) == hipErrorNotReady;
      cx.detached_lane[c] = last_still_runs && !host_link_busy ? cx.detached_lane[c] ^ 1u : 0u;
      if (cx.detached_lane[c]) s = cx.alt_streams[c];
    }
    r.stream = s;
    e = hipStreamWaitEvent(s, fork, 0);
    if (e != hipSuccess) return hip_fail(e, "hipStreamWaitEvent(fork)");
    if (dma) {
      if (timing) {
        e = hipEventRecord(r.ev_begin, s);
        if (e != hipSuccess) return hip_fail(e, "hipEventRecord(begin)");
      }
      rc = run_dma(p, plan.cls[c], chunk_bytes, c, s);
      if (rc != FT_OK) {
        put_event(p, false, fork);
        return fail_submit(p, job, rc);
      }
      if (timing) {
        e = hipEventRecord(r.ev_end, s);
        if (e != hipSuccess) return hip_fail(e, "hipEventRecord(end)");
      }
    } else {
      e = launch_copy(r.table, r.light ? kLightPoolToPool : c, r.workgroups, s, r.ev_begin, r.ev_end);
      if (e != hipSuccess) return hip_fail(e, "launch_copy");
    }
    e = hipEventRecord(r.ev_done, s);
    if (e != hipSuccess) return hip_fail(e, "hipEventRecord(done)");
    if (two_lanes) {
      std::lock_guard<std::mutex> ctx_lock(p->ctx->mu);
      e = hipEventRecord(p->ctx->lane_marker[c], s);
      if (e != hipSuccess) return hip_fail(e, "hipEventRecord(lane marker)");
    }
    if (c != FT_P2P && !dma && (flags & FT_DETACHED)) {
      // a host-link kernel that detached pool->pool launches may meet: say when it is over
      std::lock_guard<std::mutex> ctx_lock(p->ctx->mu);
      if (p->ctx->hostlink_marker == nullptr) {
        e = hipEventCreateWithFlags(&p->ctx->hostlink_marker, hipEventDisableTiming);
        if (e != hipSuccess) return hip_fail(e, "hipEventCreateWithFlags(host-link marker)");
      }
      e = hipEventRecord(p->ctx->hostlink_marker, s);
      if (e != hipSuccess) return hip_fail(e, "hipEventRecord(host-link marker)");
    }
    if (!(flags & FT_DETACHED)) {
      e = hipStreamWaitEvent(user, r.ev_done, 0);
      if (e != hipSuccess) return hip_fail(e, "hipStreamWaitEvent(join)");
    }
  }
  put_event(p, false, fork);
  return FT_OK;
}

}  // namespace ft

using namespace ft;

extern "C" {

int ft_pool_create(ft_pool **out, void *dev_base, uint64_t bytes, uint64_t slab_bytes, int device) try {
  if (out == nullptr) return FT_EINVAL;
  int rc = SlabPool::check_segment(dev_base, bytes, slab_bytes);
  if (rc != FT_OK) return rc;
  if (device < 0) return FT_EINVAL;
  ft_pool *p = new ft_pool(slab_bytes, device);
  p->slabs.add_segment(dev_base, bytes);
  *out = p;
  return FT_OK;
}
FT_CATCH_ALL

int ft_pool_grow(ft_pool *p, void *dev_base, uint64_t bytes) try {
  if (p == nullptr) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  return p->slabs.add_segment(dev_base, bytes);
}
FT_CATCH_ALL

int ft_pool_shrink(ft_pool *p, void **dev_base_out, uint64_t *bytes_out) {
  if (p == nullptr) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  return p->slabs.drop_last_segment(dev_base_out, bytes_out);
}

int ft_pool_usage(ft_pool *p, uint64_t *total_bytes_out, uint64_t *live_bytes_out) {
  if (p == nullptr) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  if (total_bytes_out) *total_bytes_out = p->slabs.total_bytes();
  if (live_bytes_out) *live_bytes_out = p->slabs.live_bytes();
  return FT_OK;
}

int ft_pool_destroy(ft_pool *p) {
  if (p == nullptr) return FT_EINVAL;
  int rc = FT_OK;
  {
    std::lock_guard<std::mutex> lock(p->mu);
    DeviceGuard guard(p->device);
    for (auto &kv : p->jobs) {
      Job *job = kv.second.get();
      if (job->open) {
        if (open_wait(p, job->open, job->id) != FT_OK) rc = FT_EHIP;
        retire(p, job);
      } else if (!job->waited) {
        if (wait_locked(p, job) != FT_OK) rc = FT_EHIP;
        else finish_staging(p, job);
      }
      release_device_side(p, job);
    }
    p->jobs.clear();  // the last job of an open sequence joins its feeder threads here
  }
  delete p;
  return rc;
}

int ft_slab_alloc(ft_pool *p, uint64_t nbytes, ft_off_t *off_out) try {
  if (p == nullptr) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  return p->slabs.alloc(nbytes, off_out);
}
FT_CATCH_ALL

int ft_slab_free(ft_pool *p, ft_off_t off) {
  if (p == nullptr) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  return p->slabs.free(off);
}

void *ft_pool_ptr(ft_pool *p, ft_off_t off) {
  if (p == nullptr) return nullptr;
  std::lock_guard<std::mutex> lock(p->mu);
  return p->slabs.ptr(off);
}

int ft_host_window_add(ft_pool *p, void *host_base, uint64_t bytes) {
  if (p == nullptr || host_base == nullptr || bytes == 0) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  p->windows.push_back(HostWindow{reinterpret_cast<uint64_t>(host_base), bytes, false});
  return FT_OK;
}

int ft_pageable_window_add(ft_pool *p, void *host_base, uint64_t bytes) {
  if (p == nullptr || host_base == nullptr || bytes == 0) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  p->windows.push_back(HostWindow{reinterpret_cast<uint64_t>(host_base), bytes, true});
  return FT_OK;
}

int ft_set_tuning(ft_pool *p, int link_class, uint32_t workgroups, uint64_t tile_bytes) {
  if (p == nullptr || link_class < 0 || link_class >= FT_NCLASS) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  p->tuning[link_class].workgroups = workgroups;
  p->tuning[link_class].tile_bytes = tile_bytes;
  return FT_OK;
}

int ft_submit_transfers(ft_pool *p, const ft_desc *descs, uint32_t ndesc, const uint32_t *weights,
                        uint32_t nfunc, uint64_t chunk_bytes, uint32_t flags, void *hip_stream,
                        ft_job_t *job_out) try {
  if (p == nullptr || job_out == nullptr) return FT_EINVAL;
  const auto t0 = std::chrono::steady_clock::now();
  std::lock_guard<std::mutex> lock(p->mu);
  SubmitPlan plan;
  int rc = plan_submit(p->slabs, p->windows, descs, ndesc, weights, nfunc, chunk_bytes, flags, &plan);
  if (rc != FT_OK) return rc;

  if ((flags & FT_OPEN) && (flags & FT_PATH_DMA)) return FT_EINVAL;
  if (plan.has_pageable && !(flags & FT_OPEN) && (flags & FT_PATH_DMA)) return FT_EINVAL;
  std::unique_ptr<Job> job(new Job());
  job->flags = flags;
  job->keep = (flags & (FT_KEEP | FT_LOG | FT_TIMING)) != 0;
  job->chunk_bytes = chunk_bytes;
  job->nfunc = nfunc;
  job->id = p->next_job;
  bool any = false;
  for (int c = 0; c < FT_NCLASS; ++c) {
    any = any || plan.cls[c].nchunks > 0;
    job->class_payload[c] = plan.cls[c].payload;
    job->class_chunks[c] = plan.cls[c].nchunks;
  }

  if (any && (flags & FT_OPEN)) {
    DeviceGuard guard(p->device);
    rc = ensure_device(p);
    if (rc != FT_OK) return rc;
    rc = open_submit(p, job.get(), plan, weights, chunk_bytes, static_cast<hipStream_t>(hip_stream));
    if (rc != FT_OK) return rc;
  } else if (any) {
    DeviceGuard guard(p->device);
    rc = ensure_device(p);
    if (rc != FT_OK) return rc;
    hipStream_t user = static_cast<hipStream_t>(hip_stream);
    if (plan.has_pageable) {
      rc = stage_closed_job(p, job.get(), plan);
      if (rc != FT_OK) return fail_submit(p, job.get(), rc);
    }
    shape_classes(p, job.get(), plan, chunk_bytes);
    bool launched = false;
    rc = launch_with_the_launch(p, job.get(), plan, chunk_bytes, flags, user, &launched);
    if (rc == FT_OK && !launched) rc = launch_with_uploaded_tables(p, job.get(), plan, chunk_bytes, flags, user);
    if (rc != FT_OK) return rc;
  }

  for (int c = 0; c < FT_NCLASS; ++c) job->run[c].plan = std::move(plan.cls[c]);
  hold_allocations(p, job.get(), plan.allocs);
  p->next_job += 1;
  *job_out = job->id;
  job->host_submit_us =
      std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t0).count();
  p->jobs[job->id] = std::move(job);
  return FT_OK;
}
FT_CATCH_ALL

int ft_submit_merge(ft_pool *p, ft_job_t open_id, const ft_desc *descs, uint32_t ndesc, const uint32_t *weights,
                    uint32_t nfunc, uint32_t flags, void *hip_stream, ft_job_t *job_out) try {
  if (p == nullptr || job_out == nullptr) return FT_EINVAL;
  if (flags & ~(uint32_t)(FT_VALIDATE | FT_KEEP)) return FT_EINVAL;
  const auto t0 = std::chrono::steady_clock::now();
  std::lock_guard<std::mutex> lock(p->mu);
  auto it = p->jobs.find(open_id);
  if (it == p->jobs.end() || !it->second->open || !(it->second->flags & FT_OPEN)) return FT_EINVAL;
  Job *open_job = it->second.get();
  SubmitPlan plan;
  int rc = plan_submit(p->slabs, p->windows, descs, ndesc, weights, nfunc, open_job->chunk_bytes, flags, &plan);
  if (rc != FT_OK) return rc;
  std::unique_ptr<Job> job(new Job());
  job->flags = flags | FT_DETACHED;
  job->keep = (flags & FT_KEEP) != 0;
  job->chunk_bytes = open_job->chunk_bytes;
  job->nfunc = nfunc;
  job->id = p->next_job;
  bool any = false;
  for (int c = 0; c < FT_NCLASS; ++c) {
    any = any || plan.cls[c].nchunks > 0;
    job->class_payload[c] = plan.cls[c].payload;
    job->class_chunks[c] = plan.cls[c].nchunks;
  }
  if (any) {
    DeviceGuard guard(p->device);
    rc = open_merge(p, open_job, job.get(), plan, weights, static_cast<hipStream_t>(hip_stream));
    if (rc != FT_OK) return rc;
  }
  hold_allocations(p, job.get(), plan.allocs);
  p->next_job += 1;
  *job_out = job->id;
  job->host_submit_us =
      std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t0).count();
  p->jobs[job->id] = std::move(job);
  return FT_OK;
}
FT_CATCH_ALL

int ft_job_reweight(ft_pool *p, ft_job_t id, const uint32_t *weights, uint32_t nfunc, void *hip_stream,
                    uint64_t *batch_out) try {
  if (p == nullptr || weights == nullptr) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  auto it = p->jobs.find(id);
  if (it == p->jobs.end() || !it->second->open || it->second->nfunc != nfunc) return FT_EINVAL;
  for (uint32_t f = 0; f < nfunc; ++f)
    if (weights[f] == 0) return FT_EINVAL;
  uint64_t batches[FT_NCLASS];
  DeviceGuard guard(p->device);
  int rc = open_reweight(p, it->second.get(), weights, static_cast<hipStream_t>(hip_stream), batches);
  if (rc != FT_OK) return rc;
  if (batch_out != nullptr)
    for (int c = 0; c < FT_NCLASS; ++c) batch_out[c] = batches[c];
  return FT_OK;
}
FT_CATCH_ALL

int ft_reserve_rings(ft_pool *p, uint64_t chunk_bytes) try {
  if (p == nullptr || chunk_bytes == 0 || chunk_bytes % 16 != 0) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  DeviceGuard guard(p->device);
  int rc = ensure_device(p);
  if (rc != FT_OK) return rc;
  const uint64_t slots = (uint64_t)((p->batch_depth ? p->batch_depth : 3) + 1) * (p->batch_chunks ? p->batch_chunks : 5);
  char *ring[2] = {nullptr, nullptr};
  uint64_t cap[2] = {0, 0};
  // both are taken before either is given back, so that they are two buffers
  for (int k = 0; k < 2 && rc == FT_OK; ++k) rc = get_pinned(p, slots * chunk_bytes, &ring[k], &cap[k]);
  for (int k = 0; k < 2; ++k) put_pinned(p, ring[k], cap[k]);
  return rc;
}
FT_CATCH_ALL

int ft_set_stage_threads(ft_pool *p, uint32_t threads) {
  if (p == nullptr || threads == 0 || threads > 64) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  p->stage_threads = threads;
  return FT_OK;
}

int ft_set_batch(ft_pool *p, uint32_t batch_chunks, uint32_t depth) {
  if (p == nullptr || batch_chunks == 0 || depth == 0) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  p->batch_chunks = batch_chunks;
  p->batch_depth = depth;
  return FT_OK;
}

int ft_timing_epoch(ft_pool *p, void *hip_stream) {
  if (p == nullptr) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  DeviceGuard guard(p->device);
  int rc = ensure_device(p);
  if (rc != FT_OK) return rc;
  hipEvent_t ev = nullptr;
  {
    std::lock_guard<std::mutex> ctx_lock(p->ctx->mu);
    ev = p->ctx->epoch;
  }
  if (ev == nullptr) FT_HIP(p, hipEventCreateWithFlags(&ev, hipEventDefault));
  FT_HIP(p, hipEventRecord(ev, static_cast<hipStream_t>(hip_stream)));
  FT_HIP(p, hipEventSynchronize(ev));
  std::lock_guard<std::mutex> ctx_lock(p->ctx->mu);
  p->ctx->epoch = ev;
  return FT_OK;
}

int ft_wait(ft_pool *p, ft_job_t id) {
  if (p == nullptr) return FT_EINVAL;
  std::unique_lock<std::mutex> lock(p->mu);
  auto it = p->jobs.find(id);
  if (it == p->jobs.end() || it->second->waited) return FT_EINVAL;
  Job *job = it->second.get();
  // Blocking happens without the pool's mutex, so that other threads can submit, merge and
  // wait meanwhile. `waited` refuses a second ft_wait on the job, `waiting` a release of it.
  job->waited = true;
  job->waiting = true;
  int rc;
  if (job->open) {
    std::shared_ptr<OpenState> st = job->open;  // the feeder threads never take the pool's mutex
    lock.unlock();
    rc = open_wait(p, st, id);
    lock.lock();
    retire(p, job);  // also after a failure: nothing of the job is in flight any more
  } else {
    hipEvent_t done[FT_NCLASS];
    for (int c = 0; c < FT_NCLASS; ++c) done[c] = job->run[c].used ? job->run[c].ev_done : nullptr;
    lock.unlock();
    {
      DeviceGuard guard(p->device);
      hipError_t e = hipSuccess;
      for (int c = 0; c < FT_NCLASS; ++c)
        if (done[c] != nullptr && hipEventSynchronize(done[c]) != hipSuccess) e = hipErrorUnknown;  // shows again below
      if (e == hipSuccess) finish_staging(p, job);  // (`waiting` keeps the record alive meanwhile)
    }
    lock.lock();
    rc = wait_locked(p, job);  // the events have fired: reads times and logs, retires
  }
  job->waiting = false;
  if (rc != FT_OK) return rc;
  if (!job->keep) {
    release_device_side(p, job);
    p->jobs.erase(id);
  }
  return FT_OK;
}

int ft_job_done(ft_pool *p, ft_job_t id, int *done_out) {
  if (p == nullptr || done_out == nullptr) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  auto it = p->jobs.find(id);
  if (it == p->jobs.end()) return FT_EINVAL;
  Job *job = it->second.get();
  *done_out = 1;
  if (job->waited) return FT_OK;
  if (job->open) {
    *done_out = open_done(job->open, id) ? 1 : 0;
    return FT_OK;
  }
  DeviceGuard guard(p->device);
  for (int c = 0; c < FT_NCLASS; ++c) {
    if (!job->run[c].used) continue;
    const hipError_t e = hipEventQuery(job->run[c].ev_done);
    if (e == hipErrorNotReady) {
      *done_out = 0;
    } else if (e != hipSuccess) {
      p->hip_error = std::string("hipEventQuery: ") + hipGetErrorString(e);
      return FT_EHIP;
    }
  }
  return FT_OK;
}

int ft_job_release(ft_pool *p, ft_job_t id) {
  if (p == nullptr) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  auto it = p->jobs.find(id);
  if (it == p->jobs.end() || !it->second->waited) return FT_EINVAL;
  if (it->second->waiting) return FT_EBUSY;  // a thread is inside ft_wait for it
  release_device_side(p, it->second.get());
  p->jobs.erase(it);
  return FT_OK;
}

int ft_job_stats(ft_pool *p, ft_job_t id, ft_job_stats_t *out) {
  if (p == nullptr || out == nullptr) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  auto it = p->jobs.find(id);
  if (it == p->jobs.end()) return FT_EINVAL;
  const Job *job = it->second.get();
  std::memset(out, 0, sizeof(*out));
  for (int c = 0; c < FT_NCLASS; ++c) {
    const ClassRun &r = job->run[c];
    ft_class_stats &s = out->cls[c];
    s.payload_bytes = job->class_payload[c];
    s.chunks = job->class_chunks[c];
    s.tickets = r.used ? r.table.ntickets : 0;
    s.tile_bytes = r.tile_bytes;
    s.workgroups = r.workgroups;
    s.in_launch = r.on_user_stream ? 1u : 0u;
    s.device_ms = r.device_ms;
    s.begin_ms = r.begin_ms;
    s.end_ms = r.end_ms;
    if (job->open && (job->flags & FT_OPEN)) {
      // the whole sequence so far, merged jobs included: tickets and kernel time of all batches
      uint64_t batches = 0;
      open_stats(job->open, c, &s.tickets, &s.tile_bytes, &s.workgroups, &s.device_ms, &batches);
    }
  }
  out->host_submit_us = job->host_submit_us;
  return FT_OK;
}

int ft_job_schedule(ft_pool *p, ft_job_t id, int link_class, uint32_t *func_out, uint32_t *chunk_out,
                    uint64_t cap, uint64_t *n_out) try {
  if (p == nullptr || n_out == nullptr || link_class < 0 || link_class >= FT_NCLASS) return FT_EINVAL;
  if (cap != 0 && (func_out == nullptr || chunk_out == nullptr)) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  auto it = p->jobs.find(id);
  if (it == p->jobs.end() || !it->second->keep) return FT_EINVAL;
  Job *job = it->second.get();
  ClassRun &r = job->run[link_class];
  *n_out = r.plan.nchunks;
  uint64_t n = r.plan.nchunks < cap ? r.plan.nchunks : cap;
  if (!r.used || n == 0) return FT_OK;
  DeviceGuard guard(p->device);
  Blob out;  // recycled like the table buffers
  int rc = get_blob(p, 2 * n * sizeof(uint32_t), false, &out);
  if (rc != FT_OK) return rc;
  uint32_t *dev = reinterpret_cast<uint32_t *>(out.dev);
  // ordered after the job's own kernel and table upload (a job that went with its launch carries its tables along)
  hipStream_t s = r.stream != nullptr ? r.stream : p->ctx->streams[link_class];
  hipError_t e = launch_decode(r.table, dev, dev + n, n, s, job->inline_tables.get());
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e == hipSuccess) e = hipMemcpy(func_out, dev, n * sizeof(uint32_t), hipMemcpyDeviceToHost);
  if (e == hipSuccess) e = hipMemcpy(chunk_out, dev + n, n * sizeof(uint32_t), hipMemcpyDeviceToHost);
  if (e != hipSuccess) (void)hipDeviceSynchronize();  // the decode may still be writing
  put_blob(p, out);
  if (e != hipSuccess) {
    p->hip_error = std::string("ft_job_schedule: ") + hipGetErrorString(e);
    return FT_EHIP;
  }
  return FT_OK;
}
FT_CATCH_ALL

int ft_job_log(ft_pool *p, ft_job_t id, int link_class, uint64_t *t_begin_ns, uint64_t *t_end_ns,
               uint32_t *func_out, uint32_t *chunk_out, uint64_t *byte_off_out, uint32_t *bytes_out, uint64_t cap,
               uint64_t *n_out) try {
  if (p == nullptr || n_out == nullptr || link_class < 0 || link_class >= FT_NCLASS) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  auto it = p->jobs.find(id);
  if (it == p->jobs.end() || !it->second->waited || it->second->waiting || !(it->second->flags & FT_LOG))
    return FT_EINVAL;
  const Job *job = it->second.get();
  const double ns_per_tick = p->ctx->clock_khz > 0 ? 1.0e6 / p->ctx->clock_khz : 10.0;
  if (job->open) {
    if (!(job->flags & FT_OPEN)) return FT_EINVAL;  // the log belongs to the sequence: ask the open job
    return open_log(job->open, link_class, ns_per_tick, t_begin_ns, t_end_ns, nullptr, func_out, chunk_out,
                    byte_off_out, bytes_out, nullptr, cap, n_out);
  }
  const ClassRun &r = job->run[link_class];
  const uint64_t nt = r.log_host.size();
  *n_out = nt;
  const ClassPlan &cp = r.plan;
  for (uint64_t t = 0; t < nt && t < cap; ++t) {
    // everything below is what the copy kernel wrote: its clock, and what its own decode made of
    // the ticket. The host only names the function (its table index -> the caller's id).
    const LogEntry &L = r.log_host[t];
    if (t_begin_ns) t_begin_ns[t] = (uint64_t)(L.t_begin * ns_per_tick);
    if (t_end_ns) t_end_ns[t] = (uint64_t)(L.t_end * ns_per_tick);
    if (func_out) func_out[t] = L.fl < cp.funcs.size() ? cp.funcs[L.fl].func : UINT32_MAX;
    if (chunk_out) chunk_out[t] = (uint32_t)L.k;
    if (byte_off_out) byte_off_out[t] = L.b0;
    if (bytes_out) bytes_out[t] = (uint32_t)(L.b1 - L.b0);
  }
  return FT_OK;
}
FT_CATCH_ALL

int ft_job_log_jobs(ft_pool *p, ft_job_t id, int link_class, uint64_t *job_out, uint32_t *batch_out, uint64_t cap,
                    uint64_t *n_out) try {
  if (p == nullptr || n_out == nullptr || link_class < 0 || link_class >= FT_NCLASS) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  auto it = p->jobs.find(id);
  if (it == p->jobs.end() || !it->second->waited || it->second->waiting || !it->second->open ||
      (it->second->flags & (FT_LOG | FT_OPEN)) != (FT_LOG | FT_OPEN))
    return FT_EINVAL;
  return open_log(it->second->open, link_class, 1.0, nullptr, nullptr, job_out, nullptr, nullptr, nullptr, nullptr,
                  batch_out, cap, n_out);
}
FT_CATCH_ALL

int ft_job_log_workgroups(ft_pool *p, ft_job_t id, int link_class, uint32_t *ticket_wg, uint64_t cap,
                          uint64_t *wg_entry_ns, uint64_t *wg_exit_ns, uint32_t wg_cap, uint32_t *nwg_out) {
  if (p == nullptr || nwg_out == nullptr || link_class < 0 || link_class >= FT_NCLASS) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  auto it = p->jobs.find(id);
  if (it == p->jobs.end() || !it->second->waited || it->second->waiting || !(it->second->flags & FT_LOG))
    return FT_EINVAL;
  if (it->second->open) return FT_EINVAL;  // an open sequence keeps the per-ticket record only
  const ClassRun &r = it->second->run[link_class];
  const double ns_per_tick = p->ctx->clock_khz > 0 ? 1.0e6 / p->ctx->clock_khz : 10.0;
  if (ticket_wg)
    for (uint64_t t = 0; t < r.log_host.size() && t < cap; ++t) ticket_wg[t] = r.log_host[t].wg;
  *nwg_out = (uint32_t)r.wg_log_host.size();
  for (uint32_t w = 0; w < r.wg_log_host.size() && w < wg_cap; ++w) {
    if (wg_entry_ns) wg_entry_ns[w] = (uint64_t)(r.wg_log_host[w].t_entry * ns_per_tick);
    if (wg_exit_ns) wg_exit_ns[w] = (uint64_t)(r.wg_log_host[w].t_exit * ns_per_tick);
  }
  return FT_OK;
}

int ft_job_log_units(ft_pool *p, ft_job_t id, int link_class, uint32_t *unit_out, uint32_t wg_cap, uint32_t *nwg_out) {
  if (p == nullptr || nwg_out == nullptr || link_class < 0 || link_class >= FT_NCLASS) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  auto it = p->jobs.find(id);
  if (it == p->jobs.end() || !it->second->waited || it->second->waiting || !(it->second->flags & FT_LOG))
    return FT_EINVAL;
  if (it->second->open) return FT_EINVAL;  // an open sequence keeps the per-ticket record only
  const ClassRun &r = it->second->run[link_class];
  *nwg_out = (uint32_t)r.wg_log_host.size();
  if (unit_out)
    for (uint32_t w = 0; w < r.wg_log_host.size() && w < wg_cap; ++w) unit_out[w] = r.wg_log_host[w].unit;
  return FT_OK;
}

int ft_job_arrival(ft_pool *p, ft_job_t id, int link_class, uint64_t *batch_out) {
  if (p == nullptr || batch_out == nullptr || link_class < 0 || link_class >= FT_NCLASS) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  auto it = p->jobs.find(id);
  if (it == p->jobs.end() || !it->second->open) return FT_EINVAL;
  return open_arrival(it->second->open, id, link_class, batch_out);
}

int ft_job_progress(ft_pool *p, ft_job_t id, int link_class, uint64_t *bytes_done, uint32_t nfunc,
                    uint64_t *batches_done) {
  if (p == nullptr || bytes_done == nullptr || link_class < 0 || link_class >= FT_NCLASS) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  auto it = p->jobs.find(id);
  if (it == p->jobs.end() || !it->second->open || it->second->nfunc != nfunc) return FT_EINVAL;
  return open_progress(it->second->open, id, link_class, bytes_done, nfunc, batches_done);
}

int ft_job_batches(ft_pool *p, ft_job_t id, int link_class, uint64_t *job_out, uint32_t *func_out,
                   uint32_t *chunk_out, uint32_t *batch_out, uint64_t cap, uint64_t *n_out) {
  if (p == nullptr || n_out == nullptr || link_class < 0 || link_class >= FT_NCLASS) return FT_EINVAL;
  if (cap != 0 && (job_out == nullptr || func_out == nullptr || chunk_out == nullptr || batch_out == nullptr))
    return FT_EINVAL;
  std::lock_guard<std::mutex> lock(p->mu);
  auto it = p->jobs.find(id);
  if (it == p->jobs.end() || !it->second->open || !(it->second->flags & FT_OPEN) ||
      !(it->second->flags & FT_KEEP))
    return FT_EINVAL;
  *n_out = open_order(it->second->open, link_class, job_out, func_out, chunk_out, batch_out, cap);
  return FT_OK;
}

int ft_slo_weights(const double *data_size, const double *l_slo, const double *l_infer, uint32_t n,
                   double bw_all, uint32_t total, double *rate_out, uint32_t *weights_out) {
  if (data_size == nullptr || l_slo == nullptr || l_infer == nullptr || weights_out == nullptr || n == 0)
    return FT_EINVAL;
  if (!(bw_all > 0.0)) return FT_EINVAL;
  if (total == 0) total = 64;
  std::vector<double> rate(n);
  double sum = 0.0;
  for (uint32_t i = 0; i < n; ++i) {
    const double slack = l_slo[i] - l_infer[i];
    if (!(slack > 0.0) || data_size[i] < 0.0) return FT_EINVAL;
    rate[i] = data_size[i] / slack;
    sum = sum + rate[i];
  }
  const double idle = bw_all - sum;
  if (idle > 0.0) {
    uint32_t tight = 0;
    for (uint32_t i = 1; i < n; ++i)
      if (l_slo[i] - l_infer[i] < l_slo[tight] - l_infer[tight]) tight = i;
    rate[tight] = rate[tight] + idle;
  }
  double s = 0.0;
  for (uint32_t i = 0; i < n; ++i) s = s + rate[i];
  for (uint32_t i = 0; i < n; ++i) {
    if (rate_out) rate_out[i] = rate[i];
    if (!(s > 0.0)) {
      weights_out[i] = 1;
      continue;
    }
    const double w = std::floor(rate[i] / s * (double)total + 0.5);
    weights_out[i] = w >= 1.0 ? (w > 4294967295.0 ? 4294967295u : (uint32_t)w) : 1u;
  }
  return FT_OK;
}

int ft_plan_schedule(const uint64_t *stream_bytes, const uint32_t *weights, uint32_t nfunc,
                     uint64_t chunk_bytes, uint32_t *func_out, uint32_t *chunk_out, uint64_t cap,
                     uint64_t *n_out) try {
  if (stream_bytes == nullptr || weights == nullptr || n_out == nullptr || nfunc == 0) return FT_EINVAL;
  if (chunk_bytes == 0 || chunk_bytes % 16 != 0) return FT_EINVAL;
  if (cap != 0 && (func_out == nullptr || chunk_out == nullptr)) return FT_EINVAL;
  std::vector<Func> funcs;
  for (uint32_t f = 0; f < nfunc; ++f) {
    if (weights[f] == 0) return FT_EINVAL;
    if (stream_bytes[f] == 0) continue;
    Func fn{};
    fn.stream_bytes = stream_bytes[f];
    fn.nchunks = stream_bytes[f] / chunk_bytes + (stream_bytes[f] % chunk_bytes != 0);
    fn.func = f;
    fn.weight = weights[f];
    funcs.push_back(fn);
  }
  std::vector<Phase> phases;
  std::vector<Slot> slots;
  uint64_t n = 0;
  int rc = build_phases(funcs, phases, slots, &n);
  if (rc != FT_OK) return rc;
  *n_out = n;
  for (uint64_t rank = 0; rank < n && rank < cap; ++rank) {
    const ChunkId id = decode_rank(phases.data(), (uint32_t)phases.size(), slots.data(), rank);
    func_out[rank] = funcs[id.fl].func;
    chunk_out[rank] = (uint32_t)id.k;
  }
  return FT_OK;
}
FT_CATCH_ALL

int ft_plan_tickets(const uint64_t *stream_bytes, const uint32_t *weights, uint32_t nfunc,
                    uint64_t chunk_bytes, uint64_t tile_bytes, uint32_t *func_out, uint32_t *chunk_out,
                    uint64_t *byte_off_out, uint32_t *bytes_out, uint64_t cap, uint64_t *n_out) try {
  if (stream_bytes == nullptr || weights == nullptr || n_out == nullptr || nfunc == 0) return FT_EINVAL;
  if (chunk_bytes == 0 || chunk_bytes % 16 != 0) return FT_EINVAL;
  if (cap != 0 && (func_out == nullptr || chunk_out == nullptr || byte_off_out == nullptr || bytes_out == nullptr))
    return FT_EINVAL;
  ClassPlan cp;
  for (uint32_t f = 0; f < nfunc; ++f) {
    if (weights[f] == 0) return FT_EINVAL;
    if (stream_bytes[f] == 0) continue;
    Func fn{};
    fn.stream_bytes = stream_bytes[f];
    fn.nchunks = stream_bytes[f] / chunk_bytes + (stream_bytes[f] % chunk_bytes != 0);
    fn.func = f;
    fn.weight = weights[f];
    cp.funcs.push_back(fn);
  }
  int rc = build_phases(cp.funcs, cp.phases, cp.slots, &cp.nchunks);
  if (rc != FT_OK) return rc;
  uint64_t tile = 0, ntickets = 0;
  uint32_t tpc = 0;
  tile_shape(chunk_bytes, tile_bytes, &tile, &tpc);
  std::vector<Skip> skips;
  build_skips(cp, chunk_bytes, tile, tpc, &skips, &ntickets);
  *n_out = ntickets;
  for (uint64_t t = 0; t < ntickets && t < cap; ++t) {
    const uint64_t v = ticket_to_tile(skips.data(), (uint32_t)skips.size(), t);
    const uint64_t rank = v / tpc, ti = v % tpc;
    const ChunkId id = decode_rank(cp.phases.data(), (uint32_t)cp.phases.size(), cp.slots.data(), rank);
    const Func &fn = cp.funcs[id.fl];
    uint64_t lo = ti * tile, hi = lo + tile;
    if (hi > chunk_bytes) hi = chunk_bytes;
    uint64_t b0 = id.k * chunk_bytes + lo, b1 = id.k * chunk_bytes + hi;
    if (b1 > fn.stream_bytes) b1 = fn.stream_bytes;
    if (b0 > b1) b0 = b1;
    func_out[t] = fn.func;
    chunk_out[t] = (uint32_t)id.k;
    byte_off_out[t] = b0;
    bytes_out[t] = (uint32_t)(b1 - b0);
  }
  return FT_OK;
}
FT_CATCH_ALL

int ft_plain_copy(void *dst, const void *src, uint64_t bytes, uint32_t workgroups, void *hip_stream) {
  if (bytes == 0) return FT_OK;
  if (dst == nullptr || src == nullptr || bytes % 16 != 0) return FT_EINVAL;
  if (reinterpret_cast<uintptr_t>(dst) % 16 != 0 || reinterpret_cast<uintptr_t>(src) % 16 != 0) return FT_EINVAL;
  hipError_t e = launch_plain_copy(dst, src, bytes, workgroups, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? FT_OK : FT_EHIP;
}

int ft_plain_read(const void *src, uint64_t bytes, uint32_t workgroups, void *hip_stream) {
  if (bytes == 0) return FT_OK;
  if (src == nullptr || bytes % 16 != 0 || reinterpret_cast<uintptr_t>(src) % 16 != 0) return FT_EINVAL;
  hipError_t e = launch_plain_read(src, bytes, workgroups, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? FT_OK : FT_EHIP;
}

int ft_plain_fill(void *dst, uint64_t bytes, uint32_t word, uint32_t workgroups, void *hip_stream) {
  if (bytes == 0) return FT_OK;
  if (dst == nullptr || bytes % 16 != 0 || reinterpret_cast<uintptr_t>(dst) % 16 != 0) return FT_EINVAL;
  hipError_t e = launch_plain_fill(dst, bytes, word, workgroups, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? FT_OK : FT_EHIP;
}

const char *ft_strerror(int rc) {
  switch (rc) {
    case FT_OK: return "ok";
    case FT_EINVAL: return "invalid argument";
    case FT_ENOMEM: return "no run of free slabs";
    case FT_ERANGE: return "range outside a live allocation or host window";
    case FT_EOVERLAP: return "a destination byte is written twice or also read";
    case FT_EBUSY: return "allocation is in use by a job that has not been waited for";
    case FT_EHIP: return "HIP runtime error";
    case FT_ECLOSED: return "the open job has triggered its last batch";
    case FT_E2BIG: return "schedule tables exceed the library's fixed device buffer";
    default: return "unknown code";
  }
}

const char *ft_last_hip_error(ft_pool *p) { return p ? p->hip_error.c_str() : ""; }

}  // extern "C"
