// The parts of the C ABI that the other host programs do not reach, on a machine without a GPU
// (built with tests/host/hip_stand_in.cpp under the address and undefined-behaviour sanitizers):
// the per-ticket log and the per-workgroup log with output arrays of exactly the size asked for,
// the device's ticket order against the host planner's, the comparison path that copies chunk piece
// by chunk piece, tuned launch shapes, pitched descriptors, growth and shrinkage of the pool, the
// job figures. Bytes are checked against a plain row-by-row copy.
// Usage: api_tour
#include <hip/hip_runtime_api.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "../../include/faastube.h"

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "FAIL %s line %d (case %d)\n", #c, __LINE__, g_case); std::abort(); } } while (0)
static int g_case = -1;
static const uint64_t KiB = 1024, MiB = 1024 * 1024;

int main() {
  const uint64_t seg_bytes = 16 * MiB, host_bytes = 16 * MiB;
  char *seg0 = nullptr, *seg1 = nullptr, *host = nullptr;
  CHECK(hipMalloc(reinterpret_cast<void **>(&seg0), seg_bytes) == hipSuccess);
  CHECK(hipMalloc(reinterpret_cast<void **>(&seg1), seg_bytes) == hipSuccess);
  CHECK(hipHostMalloc(reinterpret_cast<void **>(&host), host_bytes, 0) == hipSuccess);
  std::mt19937_64 r(5);
  for (uint64_t i = 0; i < host_bytes; i += 8) *reinterpret_cast<uint64_t *>(host + i) = r();
  std::memset(seg0, 0xA5, seg_bytes);
  std::memset(seg1, 0xA5, seg_bytes);
  ft_pool *pool = nullptr;
  CHECK(ft_pool_create(&pool, seg0, seg_bytes, 16 * KiB, 0) == FT_OK);
  CHECK(ft_host_window_add(pool, host, host_bytes / 2) == FT_OK);

  // growth on demand, shrinkage when the last segment is empty again
  ft_off_t big = 0;
  CHECK(ft_slab_alloc(pool, 12 * MiB, &big) == FT_OK);
  ft_off_t more = 0;
  CHECK(ft_slab_alloc(pool, 8 * MiB, &more) == FT_ENOMEM);
  CHECK(ft_pool_grow(pool, seg1, seg_bytes) == FT_OK);
  CHECK(ft_slab_alloc(pool, 8 * MiB, &more) == FT_OK && more == seg_bytes);
  CHECK(ft_pool_ptr(pool, more + 5) == seg1 + 5);
  void *base = nullptr;
  uint64_t bytes = 0;
  CHECK(ft_pool_shrink(pool, &base, &bytes) == FT_EBUSY);
  CHECK(ft_slab_free(pool, more) == FT_OK);
  CHECK(ft_pool_shrink(pool, &base, &bytes) == FT_OK && base == seg1 && bytes == seg_bytes);
  CHECK(ft_pool_shrink(pool, &base, &bytes) == FT_EINVAL);
  CHECK(ft_slab_free(pool, big) == FT_OK);
  uint64_t total = 0, live = 1;
  CHECK(ft_pool_usage(pool, &total, &live) == FT_OK && total == seg_bytes && live == 0);

  std::vector<char> expect(seg0, seg0 + seg_bytes), host_expect(host, host + host_bytes);
  for (g_case = 0; g_case < 60; ++g_case) {
    // a random job: three functions, pitched and plain pieces, all three classes
    const uint32_t flags = (g_case % 3 == 0 ? FT_LOG : 0) | (g_case % 3 == 1 ? FT_TIMING | FT_KEEP : FT_KEEP) |
                           (g_case % 5 == 4 ? FT_PATH_DMA : 0) | (g_case % 2 ? FT_VALIDATE : 0);
    if (g_case % 4 == 2) {
      for (int c = 0; c < FT_NCLASS; ++c) CHECK(ft_set_tuning(pool, c, 1 + r() % 40, (r() % 3) * 4096) == FT_OK);
    } else {
      for (int c = 0; c < FT_NCLASS; ++c) CHECK(ft_set_tuning(pool, c, 0, 0) == FT_OK);
    }
    std::vector<ft_desc> d;
    std::vector<ft_off_t> allocs;
    uint64_t hdst = host_bytes / 4;
    uint64_t stream[FT_NCLASS][3] = {};
    const uint32_t ndesc = 1 + r() % 6;
    for (uint32_t i = 0; i < ndesc; ++i) {
      ft_desc x{};
      x.func = (uint32_t)(r() % 3);
      x.rows = r() % 2 ? 1 : 1 + r() % 20;
      x.row_bytes = x.rows > 1 ? 1 + r() % 700 : 1 + r() % (200 * KiB);
      x.src_pitch = x.row_bytes + (r() % 2 ? r() % 40 : 0);
      x.dst_pitch = x.row_bytes + (r() % 2 ? r() % 40 : 0);
      const uint64_t es = (x.rows - 1) * x.src_pitch + x.row_bytes, ed = (x.rows - 1) * x.dst_pitch + x.row_bytes;
      const int cls = (int)(r() % 3);
      ft_off_t a = 0, b = 0;
      if (cls != FT_H2P) {
        CHECK(ft_slab_alloc(pool, es + 16, &a) == FT_OK);
        allocs.push_back(a);
        for (uint64_t k = 0; k < es + 16; ++k) seg0[a + k] = expect[a + k] = (char)r();
      }
      if (cls != FT_P2H) {
        CHECK(ft_slab_alloc(pool, ed + 16, &b) == FT_OK);
        allocs.push_back(b);
      }
      x.src_space = cls == FT_H2P ? FT_HOST : FT_POOL;
      x.dst_space = cls == FT_P2H ? FT_HOST : FT_POOL;
      x.src = cls == FT_H2P ? reinterpret_cast<uint64_t>(host + r() % (host_bytes / 4 - es)) : a + r() % 16;
      if (cls == FT_P2H) {
        x.dst = reinterpret_cast<uint64_t>(host + hdst + r() % 16);
        hdst += (ed + 47) / 16 * 16;
        CHECK(hdst < host_bytes / 2);
      } else {
        x.dst = b + r() % 16;
      }
      stream[cls][x.func] += x.row_bytes * x.rows;
      d.push_back(x);
      for (uint64_t row = 0; row < x.rows; ++row) {
        const char *src = cls == FT_H2P ? reinterpret_cast<const char *>(x.src) + row * x.src_pitch
                                        : expect.data() + x.src + row * x.src_pitch;
        char *dst = cls == FT_P2H ? host_expect.data() + (reinterpret_cast<char *>(x.dst) - host) + row * x.dst_pitch
                                  : expect.data() + x.dst + row * x.dst_pitch;
        std::memmove(dst, src, x.row_bytes);
      }
    }
    const uint32_t w[3] = {1 + (uint32_t)(r() % 5), 1 + (uint32_t)(r() % 5), 1 + (uint32_t)(r() % 5)};
    const uint64_t C = (uint64_t[]){64, 4096, 64 * KiB, 1 * MiB}[r() % 4];
    ft_job_t job = 0;
    CHECK(ft_submit_transfers(pool, d.data(), (uint32_t)d.size(), w, 3, C, flags, nullptr, &job) == FT_OK);
    CHECK(ft_wait(pool, job) == FT_OK);
    CHECK(std::memcmp(seg0, expect.data(), seg_bytes) == 0);
    CHECK(std::memcmp(host, host_expect.data(), host_bytes) == 0);
    ft_job_stats_t st{};
    CHECK(ft_job_stats(pool, job, &st) == FT_OK);
    for (int c = 0; c < FT_NCLASS; ++c) {
      CHECK(st.cls[c].payload_bytes == stream[c][0] + stream[c][1] + stream[c][2]);
      // the order the device uses is the order the host planner states for these stream sizes
      uint64_t n = 0, n2 = 0;
      CHECK(ft_job_schedule(pool, job, c, nullptr, nullptr, 0, &n) == FT_OK && n == st.cls[c].chunks);
      std::vector<uint32_t> f1(n), k1(n), f2(n), k2(n);
      CHECK(ft_job_schedule(pool, job, c, f1.data(), k1.data(), n, &n) == FT_OK);
      CHECK(ft_plan_schedule(stream[c], w, 3, C, f2.data(), k2.data(), n, &n2) == FT_OK && n2 == n);
      CHECK(f1 == f2 && k1 == k2);
      if ((flags & FT_LOG) && !(flags & FT_PATH_DMA) && n > 0) {
        uint64_t nt = 0;
        CHECK(ft_job_log(pool, job, c, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, &nt) == FT_OK && nt == st.cls[c].tickets);
        std::vector<uint64_t> tb(nt), te(nt);
        std::vector<uint64_t> lo(nt);
        std::vector<uint32_t> lf(nt), lk(nt), lb(nt), wg(nt);
        CHECK(ft_job_log(pool, job, c, tb.data(), te.data(), lf.data(), lk.data(), lo.data(), lb.data(), nt, &nt) == FT_OK);
        uint64_t sum = 0;
        for (uint64_t t = 0; t < nt; ++t) {
          CHECK(te[t] >= tb[t] && lb[t] > 0 && lf[t] < 3);
          CHECK(lo[t] / C == lk[t] && (lo[t] + lb[t] - 1) / C == lk[t]);  // the tile lies inside its chunk
          sum += lb[t];
        }
        CHECK(sum == st.cls[c].payload_bytes);
        uint32_t nwg = 0;
        CHECK(ft_job_log_workgroups(pool, job, c, nullptr, 0, nullptr, nullptr, 0, &nwg) == FT_OK && nwg == st.cls[c].workgroups);
        std::vector<uint64_t> t_in(nwg), t_out(nwg);
        CHECK(ft_job_log_workgroups(pool, job, c, wg.data(), nt, t_in.data(), t_out.data(), nwg, &nwg) == FT_OK);
        std::vector<uint32_t> units(nwg);  // exactly as many as promised
        CHECK(ft_job_log_units(pool, job, c, units.data(), nwg, &nwg) == FT_OK && nwg == st.cls[c].workgroups);
        for (uint64_t t = 0; t < nt; ++t) CHECK(wg[t] < nwg);
      }
    }
    CHECK(ft_job_release(pool, job) == FT_OK);
    for (ft_off_t a : allocs) CHECK(ft_slab_free(pool, a) == FT_OK);
  }
  g_case = -1;
  {
    // The store while a consumer's transfer that has not been waited for still reads a result: the result
    // cannot be moved out (FT_EBUSY), it stays where it is and no spill space is taken; once the transfer
    // has been waited for the same put goes through, the move is not waited for by the call that starts
    // it, and ft_store_get waits for the one result it returns.
    char *spill = host + host_bytes / 2;
    ft_store *store = nullptr;
    CHECK(ft_store_create(&store, pool, spill, host_bytes / 2, 6 * MiB, 256 * KiB, nullptr) == FT_OK);
    ft_off_t a = 0, b = 0, c = 0;
    CHECK(ft_store_put(store, 1, 4 * MiB, 5, &a) == FT_OK);
    std::memset(static_cast<char *>(ft_pool_ptr(pool, a)), 0x11, 4 * MiB);
    ft_desc d{};
    d.src_space = FT_POOL;
    d.dst_space = FT_HOST;
    d.src = a;
    d.dst = reinterpret_cast<uint64_t>(host);
    d.row_bytes = 64 * KiB;
    d.rows = 1;
    const uint32_t w = 1;
    ft_job_t consumer = 0;
    CHECK(ft_submit_transfers(pool, &d, 1, &w, 1, 64 * KiB, 0, nullptr, &consumer) == FT_OK);
    ft_store_stats_t st{};
    CHECK(ft_store_put(store, 2, 4 * MiB, 1, &b) == FT_EBUSY);
    CHECK(ft_store_stats(store, &st) == FT_OK && st.spill_used_bytes == 0 && st.moved_out == 0 && st.objects == 1 &&
          st.resident_bytes == 4 * MiB && st.moves_in_flight == 0);
    CHECK(ft_wait(pool, consumer) == FT_OK);
    CHECK(ft_store_put(store, 2, 4 * MiB, 1, &b) == FT_OK && b == a);  // the slabs that result 1 left, at once
    CHECK(ft_store_stats(store, &st) == FT_OK && st.spill_used_bytes == 4 * MiB && st.moved_out == 1 &&
          st.moves_in_flight == 1 && st.resident_bytes == 4 * MiB);
    std::memset(static_cast<char *>(ft_pool_ptr(pool, b)), 0x22, 4 * MiB);
    uint32_t was_out = 0;
    CHECK(ft_store_get(store, 2, &c, &was_out) == FT_OK && c == b && was_out == 0);
    CHECK(ft_store_done(store, 2) == FT_OK);  // result 1 comes back, nobody waits for it here
    CHECK(ft_store_stats(store, &st) == FT_OK && st.moved_in == 1 && st.moves_in_flight == 1 && st.spill_used_bytes == 0);
    CHECK(ft_store_get(store, 1, &c, &was_out) == FT_OK && was_out == 0);
    CHECK(ft_store_stats(store, &st) == FT_OK && st.moves_in_flight == 0 && st.stalls == 0);
    for (uint64_t i = 0; i < 4 * MiB; i += 4099) CHECK(static_cast<unsigned char *>(ft_pool_ptr(pool, c))[i] == 0x11);
    CHECK(ft_store_done(store, 1) == FT_OK);
    CHECK(ft_store_sync(store) == FT_OK);
    CHECK(ft_store_destroy(store) == FT_OK);
  }
  CHECK(ft_pool_destroy(pool) == FT_OK);
  std::printf("api_tour done\n");
  return 0;
}
