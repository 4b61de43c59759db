// Error paths of the library's host code, on a machine without a GPU: built with
// tests/host/hip_stand_in.cpp, which can make the n-th call of a runtime function (or of the kernel
// launch) fail. For every such point and n = 1, 2, ... a closed job on each launch route, an open
// job, a merge and a weight change are attempted. Whatever fails, the calls must return FT_OK or
// a negative code (never hang, never crash), nothing may stay busy afterwards (every allocation
// can be freed once the jobs that were accepted have been waited for), and the same jobs run
// again without a failure must put every byte where memcpy puts it.
// Usage: fault_paths
#include <hip/hip_runtime_api.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/faastube.h"

extern "C" int stand_in_fail(const char *name, int nth);

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "FAIL %s line %d (point %s, n %d)\n", #c, __LINE__, g_point, g_n); std::abort(); } } while (0)
static const char *g_point = "-";
static int g_n = 0;

static const uint64_t KiB = 1024, MiB = 1024 * 1024;

struct World {
  char *dev = nullptr, *host = nullptr;
  uint64_t pool_bytes = 64 * MiB, host_bytes = 32 * MiB;
  std::vector<char> expect;
  std::vector<char> pageable, pageable_expect;  // ordinary host memory for the jobs that stage
  ft_pool *pool = nullptr;
  std::vector<ft_off_t> allocs;
};

static ft_off_t alloc(World &w, uint64_t n) {
  ft_off_t off = 0;
  CHECK(ft_slab_alloc(w.pool, n, &off) == FT_OK);
  w.allocs.push_back(off);
  return off;
}

// One job of `nfunc` functions moving `bytes` each host->pool (and pool->pool when mixed); its
// expected effect is written into w.expect only when `count` (the job was accepted).
struct JobSpec {
  std::vector<ft_desc> d;
  std::vector<uint32_t> wts;
};

static JobSpec make_job(World &w, uint32_t nfunc, uint64_t bytes, bool mixed, uint64_t salt) {
  JobSpec j;
  for (uint32_t f = 0; f < nfunc; ++f) {
    ft_desc d{};
    d.func = f;
    d.rows = 1;
    d.row_bytes = bytes + f * 16 + 3;
    d.src_pitch = d.dst_pitch = d.row_bytes;
    d.dst_space = FT_POOL;
    d.dst = alloc(w, d.row_bytes + 32) + 5;
    if (mixed && f % 2 == 1) {
      const ft_off_t s = alloc(w, d.row_bytes + 32);
      std::memcpy(w.dev + s, w.host + (salt * 4099 + f * 77) % (w.host_bytes / 2), d.row_bytes + 32);
      std::memcpy(w.expect.data() + s, w.dev + s, d.row_bytes + 32);
      d.src_space = FT_POOL;
      d.src = s + 1;
    } else {
      d.src_space = FT_HOST;
      d.src = reinterpret_cast<uint64_t>(w.host + (salt * 8191 + f * 131) % (w.host_bytes / 2));
    }
    j.d.push_back(d);
    j.wts.push_back(1 + f % 3);
  }
  return j;
}

static void expect_job(World &w, const JobSpec &j) {
  for (const ft_desc &d : j.d) {
    const char *src = d.src_space == FT_POOL ? w.expect.data() + d.src : reinterpret_cast<const char *>(d.src);
    std::memmove(w.expect.data() + d.dst, src, d.row_bytes);
  }
}

// One pass over all kinds of job. inject: arm the failure before the pass.
static int pass(World &w, bool inject, const char *point, int n) {
  int failures = 0;
  std::vector<ft_job_t> to_wait;
  auto outcome = [&](int rc, const JobSpec &j, ft_job_t id) {
    CHECK(rc <= 0);
    if (rc == FT_OK) {
      expect_job(w, j);
      to_wait.push_back(id);
    } else {
      failures += 1;
    }
  };
  if (inject) CHECK(stand_in_fail(point, n) == 0);
  // closed jobs: tables inside the launch, a counter pair, uploaded tables (two classes)
  for (int kind = 0; kind < 3; ++kind) {
    JobSpec j = make_job(w, kind == 2 ? 4 : 1, kind == 0 ? 20 * KiB : 3 * MiB, kind == 2, 11 + kind);
    ft_job_t id = 0;
    const int rj = ft_submit_transfers(w.pool, j.d.data(), (uint32_t)j.d.size(), j.wts.data(), (uint32_t)j.wts.size(),
                                       256 * KiB, FT_KEEP, nullptr, &id);
    outcome(rj, j, id);
  }
  // a closed job with pageable memory on both sides (a pinned buffer of its own, copies in ft_wait)
  {
    const uint64_t n = 100 * KiB + 7;
    const ft_off_t in = alloc(w, n + 16), out = alloc(w, n + 16);
    std::memcpy(w.dev + out, w.host + 12345, n);
    std::memcpy(w.expect.data() + out, w.dev + out, n);
    ft_desc d2[2] = {};
    d2[0].func = 0; d2[0].src_space = FT_PAGEABLE; d2[0].src = reinterpret_cast<uint64_t>(w.pageable.data() + 100);
    d2[0].dst_space = FT_POOL; d2[0].dst = in + 3; d2[0].row_bytes = n; d2[0].rows = 1;
    d2[1].func = 0; d2[1].src_space = FT_POOL; d2[1].src = out;
    d2[1].dst_space = FT_PAGEABLE; d2[1].dst = reinterpret_cast<uint64_t>(w.pageable.data() + 2 * MiB + 5); d2[1].row_bytes = n; d2[1].rows = 1;
    const uint32_t one = 1;
    ft_job_t id = 0;
    const int rj = ft_submit_transfers(w.pool, d2, 2, &one, 1, 64 * KiB, FT_KEEP, nullptr, &id);
    CHECK(rj <= 0);
    if (rj == FT_OK) {
      std::memcpy(w.expect.data() + in + 3, w.pageable.data() + 100, n);
      std::memcpy(w.pageable_expect.data() + 2 * MiB + 5, w.expect.data() + out, n);
      to_wait.push_back(id);
    } else {
      failures += 1;
    }
  }
  // an open job, a merge into it, a change of its weights
  JobSpec open = make_job(w, 3, 2 * MiB, true, 29);
  ft_job_t open_id = 0;
  int rc = ft_submit_transfers(w.pool, open.d.data(), (uint32_t)open.d.size(), open.wts.data(), (uint32_t)open.wts.size(),
                               128 * KiB, FT_OPEN | FT_KEEP, nullptr, &open_id);
  outcome(rc, open, open_id);
  if (rc == FT_OK) {
    JobSpec late = make_job(w, 2, 600 * KiB, false, 31);
    ft_job_t late_id = 0;
    int rm = ft_submit_merge(w.pool, open_id, late.d.data(), (uint32_t)late.d.size(), late.wts.data(), (uint32_t)late.wts.size(),
                             FT_KEEP, nullptr, &late_id);
    if (rm == FT_ECLOSED) {
      rm = ft_submit_transfers(w.pool, late.d.data(), (uint32_t)late.d.size(), late.wts.data(), (uint32_t)late.wts.size(), 128 * KiB,
                               FT_KEEP, nullptr, &late_id);
    }
    outcome(rm, late, late_id);
    const uint32_t nw[3] = {5, 1, 2};
    const int rr = ft_job_reweight(w.pool, open_id, nw, 3, nullptr, nullptr);
    CHECK(rr <= 0);
    if (rr != FT_OK) failures += 1;
  }
  stand_in_fail(point, 0);
  // every accepted job comes to an end; a wait may report the failure of a batch
  bool data_defined = true;
  for (ft_job_t id : to_wait) {
    const int rw = ft_wait(w.pool, id);
    CHECK(rw <= 0);
    if (rw != FT_OK) {
      failures += 1;
      data_defined = false;  // some chunks of that sequence were never moved
    }
    const int rl = ft_job_release(w.pool, id);
    if (rl != FT_OK) std::fprintf(stderr, "release of job %llu -> %d (wait gave %d)\n", (unsigned long long)id, rl, rw);
    CHECK(rl == FT_OK);
  }
  // nothing is left busy
  for (ft_off_t off : w.allocs) CHECK(ft_slab_free(w.pool, off) == FT_OK);
  w.allocs.clear();
  uint64_t total = 0, live = 1;
  CHECK(ft_pool_usage(w.pool, &total, &live) == FT_OK && live == 0);
  if (data_defined) {
    CHECK(std::memcmp(w.dev, w.expect.data(), w.pool_bytes) == 0);
    CHECK(w.pageable == w.pageable_expect);
  } else {
    std::memcpy(w.expect.data(), w.dev, w.pool_bytes);  // start the next pass from what is there
    w.pageable_expect = w.pageable;
  }
  return failures;
}

int main() {
  World w;
  CHECK(hipMalloc(reinterpret_cast<void **>(&w.dev), w.pool_bytes) == hipSuccess);
  CHECK(hipHostMalloc(reinterpret_cast<void **>(&w.host), w.host_bytes, 0) == hipSuccess);
  for (uint64_t i = 0; i < w.host_bytes; ++i) w.host[i] = (char)(i * 2654435761u >> 13);
  std::memset(w.dev, 0, w.pool_bytes);
  w.expect.assign(w.pool_bytes, 0);
  CHECK(ft_pool_create(&w.pool, w.dev, w.pool_bytes, 64 * KiB, 0) == FT_OK);
  CHECK(ft_host_window_add(w.pool, w.host, w.host_bytes) == FT_OK);
  w.pageable.assign(4 * MiB, 0);
  for (uint64_t i = 0; i < 1 * MiB; ++i) w.pageable[i] = (char)(i * 40503u >> 7);
  w.pageable_expect = w.pageable;
  CHECK(ft_pageable_window_add(w.pool, w.pageable.data(), w.pageable.size()) == FT_OK);
  CHECK(pass(w, false, "-", 0) == 0);  // also creates the per-device resources
  const char *points[] = {"hipMemcpyAsync", "hipEventRecord", "hipStreamWaitEvent", "hipEventCreateWithFlags",
                          "hipMalloc",      "hipHostMalloc",  "hipEventSynchronize", "launch_copy"};
  int hit = 0;
  for (const char *point : points)
    for (int n = 1; n <= 12; ++n) {
      g_point = point;
      g_n = n;
      const int failures = pass(w, true, point, n);
      hit += failures > 0;
      g_point = "-";
      CHECK(pass(w, false, "-", 0) == 0);  // and everything works again afterwards
    }
  std::fprintf(stderr, "%d of %d injected failures were met by a call\n", hit, (int)(sizeof(points) / sizeof(points[0])) * 12);
  CHECK(hit >= 30);
  CHECK(ft_pool_destroy(w.pool) == FT_OK);
  std::printf("fault_paths done\n");
  return 0;
}
