// TEST INFRASTRUCTURE ONLY: a stand-in for the HIP runtime and for the library's kernels, so that
// the library's host code (planning, jobs, feeder threads, merges, weight changes, the staging ring,
// the store) can run on a machine without a GPU under the thread and address sanitizers. It is
// linked into a test program in place of libamdhip64 and ft_kernels.hip; it is never part of
// libfaastube.so, which has no CPU path.
//
// "Device" memory is host memory. Every stream operation is carried out at once by the calling
// thread: copies are memcpy, events are always complete, and a kernel launch walks the launch's
// tickets one after the other - ticket -> tile -> (function, chunk) -> descriptor -> pieces, read
// from the same tables the GPU kernel reads - and moves the bytes with memcpy. The order in which
// tickets move bytes does not matter for a valid job, so the result is the GPU's.
#include <hip/hip_runtime_api.h>

#include <atomic>
#include <cstdlib>
#include <cstring>

#include "../../paper_2411_01830_amd/csrc/ft_kernels.h"
#include "../../paper_2411_01830_amd/csrc/ft_tables.h"

// Failure injection for tests of the error paths: stand_in_fail("hipMemcpyAsync", 3) makes the
// third call from now of that function fail once (0 clears it). Names: the HIP calls below that
// say FAIL_POINT, and "launch_copy".
namespace {
struct FailPoint {
  const char *name;
  std::atomic<int> countdown{0};
};
FailPoint g_fail[] = {{"hipMemcpyAsync"}, {"hipEventRecord"}, {"hipStreamWaitEvent"}, {"hipEventCreateWithFlags"},
                      {"hipMalloc"},      {"hipHostMalloc"},  {"hipEventSynchronize"}, {"launch_copy"}};
bool fails_now(const char *name) {
  for (FailPoint &f : g_fail)
    if (std::strcmp(f.name, name) == 0) {
      int c = f.countdown.load();
      while (c > 0 && !f.countdown.compare_exchange_weak(c, c - 1)) {
      }
      return c == 1;
    }
  return false;
}
}  // namespace
#define FAIL_POINT(name, err) \
  if (fails_now(name)) return err

extern "C" int stand_in_fail(const char *name, int nth) {
  for (FailPoint &f : g_fail)
    if (std::strcmp(f.name, name) == 0) {
      f.countdown.store(nth);
      return 0;
    }
  return -1;
}

extern "C" {

hipError_t hipGetDeviceCount(int *count) { *count = 1; return hipSuccess; }
hipError_t hipGetDevice(int *device) { *device = 0; return hipSuccess; }
hipError_t hipSetDevice(int) { return hipSuccess; }
hipError_t hipDeviceGetAttribute(int *value, hipDeviceAttribute_t attr, int) {
  *value = attr == hipDeviceAttributeMultiprocessorCount ? 256 : 100000;
  return hipSuccess;
}
hipError_t hipDeviceSynchronize(void) { return hipSuccess; }
const char *hipGetErrorString(hipError_t) { return "stand-in"; }
hipError_t hipGetLastError(void) { return hipSuccess; }

hipError_t hipStreamCreate(hipStream_t *s) { *s = reinterpret_cast<hipStream_t>(std::malloc(8)); return hipSuccess; }
hipError_t hipStreamCreateWithFlags(hipStream_t *s, unsigned) { return hipStreamCreate(s); }
hipError_t hipStreamDestroy(hipStream_t s) { std::free(s); return hipSuccess; }
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t, unsigned) {
  FAIL_POINT("hipStreamWaitEvent", hipErrorUnknown);
  return hipSuccess;
}

hipError_t hipEventCreateWithFlags(hipEvent_t *e, unsigned) {
  FAIL_POINT("hipEventCreateWithFlags", hipErrorOutOfMemory);
  *e = reinterpret_cast<hipEvent_t>(std::malloc(8));
  return hipSuccess;
}
hipError_t hipEventRecord(hipEvent_t, hipStream_t) {
  FAIL_POINT("hipEventRecord", hipErrorUnknown);
  return hipSuccess;
}
hipError_t hipEventSynchronize(hipEvent_t) {
  FAIL_POINT("hipEventSynchronize", hipErrorUnknown);
  return hipSuccess;
}
hipError_t hipEventQuery(hipEvent_t) { return hipSuccess; }
hipError_t hipEventElapsedTime(float *ms, hipEvent_t, hipEvent_t) { *ms = 0.001f; return hipSuccess; }

hipError_t hipMalloc(void **p, size_t n) {
  FAIL_POINT("hipMalloc", hipErrorOutOfMemory);
  *p = std::aligned_alloc(4096, (n + 4095) / 4096 * 4096);
  return *p ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipHostMalloc(void **p, size_t n, unsigned) {
  FAIL_POINT("hipHostMalloc", hipErrorOutOfMemory);
  *p = std::aligned_alloc(4096, (n + 4095) / 4096 * 4096);
  return *p ? hipSuccess : hipErrorOutOfMemory;
}
hipError_t hipFree(void *p) { std::free(p); return hipSuccess; }
hipError_t hipHostFree(void *p) { std::free(p); return hipSuccess; }
hipError_t hipMemset(void *p, int v, size_t n) { std::memset(p, v, n); return hipSuccess; }
hipError_t hipMemcpy(void *d, const void *s, size_t n, hipMemcpyKind) { std::memcpy(d, s, n); return hipSuccess; }
hipError_t hipMemcpyAsync(void *d, const void *s, size_t n, hipMemcpyKind, hipStream_t) {
  FAIL_POINT("hipMemcpyAsync", hipErrorUnknown);
  std::memcpy(d, s, n);
  return hipSuccess;
}
hipError_t hipMemcpy2DAsync(void *d, size_t dp, const void *s, size_t sp, size_t w, size_t h, hipMemcpyKind, hipStream_t) {
  for (size_t r = 0; r < h; ++r) std::memcpy(static_cast<char *>(d) + r * dp, static_cast<const char *>(s) + r * sp, w);
  return hipSuccess;
}

}  // extern "C"

namespace ft {

namespace {

// The tables of a launch as ordinary pointers (a small job's lie in the blob that came with it).
struct Tables {
  const Phase *phases;
  const Slot *slots;
  const Func *funcs;
  const Xfer *xfers;
  const Skip *skips;
  const uint32_t *chunk_desc;
};

Tables tables_of(const ClassTable &T, const InlineBlob *blob) {
  const uintptr_t base = T.inline_tables ? reinterpret_cast<uintptr_t>(blob) : 0;
  Tables t;
  t.phases = reinterpret_cast<const Phase *>(base + reinterpret_cast<uintptr_t>(T.phases));
  t.slots = reinterpret_cast<const Slot *>(base + reinterpret_cast<uintptr_t>(T.slots));
  t.funcs = reinterpret_cast<const Func *>(base + reinterpret_cast<uintptr_t>(T.funcs));
  t.xfers = reinterpret_cast<const Xfer *>(base + reinterpret_cast<uintptr_t>(T.xfers));
  t.skips = reinterpret_cast<const Skip *>(base + reinterpret_cast<uintptr_t>(T.skips));
  t.chunk_desc = T.chunk_desc ? reinterpret_cast<const uint32_t *>(base + reinterpret_cast<uintptr_t>(T.chunk_desc)) : nullptr;
  return t;
}

// Bytes [p, p + n) of a descriptor's payload (row major), moved row piece by row piece.
void move_payload(const Xfer &X, uint64_t p, uint64_t n) {
  while (n > 0) {
    const uint64_t r = p / X.row_bytes, c = p % X.row_bytes;
    const uint64_t take = n < X.row_bytes - c ? n : X.row_bytes - c;
    std::memcpy(reinterpret_cast<char *>(X.dst + r * X.dst_pitch + c), reinterpret_cast<const char *>(X.src + r * X.src_pitch + c),
                take);
    p += take;
    n -= take;
  }
}

std::atomic<uint64_t> g_clock{1};

}  // namespace

hipError_t launch_copy(const ClassTable &T, int, uint32_t workgroups, hipStream_t, hipEvent_t, hipEvent_t,
                       const InlineBlob *blob) {
  if (workgroups == 0 || (T.inline_tables != 0) != (blob != nullptr)) return hipErrorInvalidValue;
  FAIL_POINT("launch_copy", hipErrorLaunchFailure);
  const Tables tb = tables_of(T, blob);
  if (T.log)
    for (uint32_t g = 0; g < workgroups; ++g) {
      T.wg_log[g].t_entry = g_clock++;
      T.wg_log[g].unit = g % 256;
    }
  for (uint64_t t = T.ticket_base; t < T.ntickets; ++t) {
    uint64_t rank, ti, b0, b1, c0;  // c0: stream offset of the chunk's first byte
    uint32_t x = 0, log_fl = 0;
    uint64_t log_k = 0;
    if (T.single) {
      rank = t / T.tiles_per_chunk;
      ti = t % T.tiles_per_chunk;
      const uint64_t stream_bytes = tb.xfers[0].row_bytes * tb.xfers[0].rows;
      uint64_t lo = ti * T.tile_bytes, hi = lo + T.tile_bytes;
      if (hi > T.chunk_bytes) hi = T.chunk_bytes;
      c0 = rank * T.chunk_bytes;
      b0 = c0 + lo;
      b1 = c0 + hi;
      if (b1 > stream_bytes) b1 = stream_bytes;
      log_k = rank;
    } else {
      const uint64_t v = ticket_to_tile(tb.skips, T.nskips, t);
      rank = v / T.tiles_per_chunk;
      ti = v % T.tiles_per_chunk;
      const ChunkId id = decode_rank(tb.phases, T.nphases, tb.slots, rank);
      const uint32_t fl = id.fl;
      const Func &f = tb.funcs[fl];
      uint32_t x0, x1;
      if (tb.chunk_desc != nullptr) {
        const uint64_t per = T.desc_per;
        const uint64_t e = ((uint64_t)f.chunk_off - fl + id.k) * per + fl + (per > 1 ? ti : 0);
        x0 = tb.chunk_desc[e];
        x1 = per > 1 ? x0 : tb.chunk_desc[e + 1];
      } else {
        x0 = f.desc_off;
        x1 = x0 + f.ndesc - 1;
      }
      c0 = (f.chunk_base + id.k) * T.chunk_bytes;
      log_fl = fl;
      log_k = f.chunk_base + id.k;
      uint64_t lo = ti * T.tile_bytes, hi = lo + T.tile_bytes;
      if (hi > T.chunk_bytes) hi = T.chunk_bytes;
      b0 = c0 + lo;
      b1 = c0 + hi;
      if (b1 > f.stream_bytes) b1 = f.stream_bytes;
      if (b0 < b1) x = x0 == x1 ? x0 : find_xfer(tb.xfers, x0, x1, b0);
    }
    const uint64_t begin = g_clock++;
    if (b0 < b1) {
      // where stream byte 0 of this function would lie if the chunk's ring slot went on for ever
      const uint64_t stage = T.stage_base + (T.stage_slot0 + (rank - T.stage_rank0)) * T.chunk_bytes - c0;
      for (uint64_t pos = b0; pos < b1; ++x) {
        Xfer X = tb.xfers[x];
        if (X.staged & kStagedSrc) {
          X.src = stage + X.stream_off;
          X.src_pitch = X.row_bytes;
        }
        if (X.staged & kStagedDst) {
          X.dst = stage + X.stream_off;
          X.dst_pitch = X.row_bytes;
        }
        const uint64_t p = pos - X.stream_off;
        uint64_t take = X.row_bytes * X.rows - p;
        if (take > b1 - pos) take = b1 - pos;
        move_payload(X, p, take);
        pos += take;
      }
    }
    if (T.log) {
      T.log[t].t_begin = begin;
      T.log[t].t_end = g_clock++;
      T.log[t].wg = (uint32_t)((t - T.ticket_base) % workgroups);
      T.log[t].fl = log_fl;
      T.log[t].k = log_k;
      T.log[t].b0 = b0;
      T.log[t].b1 = b1;
    }
  }
  if (T.log)
    for (uint32_t g = 0; g < workgroups; ++g) T.wg_log[g].t_exit = g_clock++;
  return hipSuccess;
}

hipError_t launch_decode(const ClassTable &T, uint32_t *func_out, uint32_t *chunk_out, uint64_t cap, hipStream_t,
                         const InlineBlob *blob) {
  if ((T.inline_tables != 0) != (blob != nullptr)) return hipErrorInvalidValue;
  const Tables tb = tables_of(T, blob);
  for (uint64_t rank = 0; rank < T.nchunks && rank < cap; ++rank) {
    const ChunkId id = decode_rank(tb.phases, T.nphases, tb.slots, rank);
    func_out[rank] = tb.funcs[id.fl].func;
    chunk_out[rank] = (uint32_t)(tb.funcs[id.fl].chunk_base + id.k);
  }
  return hipSuccess;
}

hipError_t launch_plain_copy(void *dst, const void *src, uint64_t bytes, uint32_t, hipStream_t) {
  std::memcpy(dst, src, bytes);
  return hipSuccess;
}

hipError_t launch_plain_read(const void *, uint64_t, uint32_t, hipStream_t) { return hipSuccess; }

hipError_t launch_plain_fill(void *dst, uint64_t bytes, uint32_t word, uint32_t, hipStream_t) {
  for (uint64_t i = 0; i + 4 <= bytes; i += 4) std::memcpy(static_cast<char *>(dst) + i, &word, 4);
  return hipSuccess;
}

}  // namespace ft
