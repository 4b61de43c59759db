// A consumer of the C ABI without Python: links libfaastube.so, owns its memory through the HIP
// runtime alone, and drives the engine from several threads at once - an open job (host->pool and
// pool->pool functions, one function from pageable memory and one to it) that two threads merge
// later jobs into while a third keeps changing its weights, closed jobs of three sizes (tables
// inside the launch, a recycled counter pair, uploaded tables), then the store. Every transfer is
// one contiguous piece, so what the pool and the pageable memory must hold is what memcpy puts into
// host images of them; both are compared whole after every round.
// Built by paper_2411_01830_amd/build.py (build_native_tests); run by tests/test_gpu_native.py.
// The library's host sources can also be compiled with -Xarch_host -fsanitize=address and linked
// into this program in place of the shared library: the address sanitizer then watches the feeder
// threads, the table generations and the recycled buffers while the GPU does the real work.
// With tests/host/hip_stand_in.cpp in place of the HIP runtime and the kernels the same program runs
// on a machine without a GPU, under the thread sanitizer (tests/test_host_logic.py does that, at a
// sixteenth of the sizes).
// Usage: c_abi_stress [rounds] [divide all sizes by]
#include <hip/hip_runtime_api.h>
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <thread>
#include <vector>
#include "../../include/faastube.h"
#define OK(c) do { int rc_ = (c); if (rc_ != 0) { std::fprintf(stderr, "FAIL %s -> %d line %d\n", #c, rc_, __LINE__); std::abort(); } } while (0)
#define HIPOK(c) do { hipError_t e_ = (c); if (e_ != hipSuccess) { std::fprintf(stderr, "HIP FAIL %s -> %s line %d\n", #c, hipGetErrorString(e_), __LINE__); std::abort(); } } while (0)

static uint64_t MiB = 1ull << 20;  // divided by the second argument: "MiB" is then the unit of all sizes

int main(int argc, char **argv) {
  const int rounds = argc > 1 ? atoi(argv[1]) : 6;
  if (argc > 2 && atoi(argv[2]) > 1) MiB /= (uint64_t)atoi(argv[2]);
  const uint64_t pool_bytes = 1024 * MiB, host_bytes = 512 * MiB;
  char *dev = nullptr, *host = nullptr;
  HIPOK(hipMalloc(&dev, pool_bytes));
  HIPOK(hipHostMalloc(&host, host_bytes, hipHostMallocDefault));
  std::mt19937_64 r(7);
  for (uint64_t i = 0; i < host_bytes / 2; i += 8) *reinterpret_cast<uint64_t *>(host + i) = r();
  std::vector<char> expect(pool_bytes, 0);
  HIPOK(hipMemset(dev, 0, pool_bytes));
  // ordinary host memory for the two functions that go through the pinned ring
  const uint64_t page_bytes = 64 * MiB;
  std::vector<char> pageable(page_bytes), pageable_expect;
  for (uint64_t i = 0; i < page_bytes / 2; i += 8) *reinterpret_cast<uint64_t *>(pageable.data() + i) = r();
  pageable_expect = pageable;
  ft_pool *pool = nullptr;
  OK(ft_pool_create(&pool, dev, pool_bytes, 64 * 1024, 0));
  OK(ft_host_window_add(pool, host, host_bytes));
  OK(ft_pageable_window_add(pool, pageable.data(), page_bytes));
  hipStream_t stream;
  HIPOK(hipStreamCreate(&stream));
  for (int round = 0; round < rounds; ++round) {
    std::fprintf(stderr, "round %d\n", round);
    OK(ft_set_batch(pool, 1 + round % 5, 1 + round % 3));
    // open job: 4 functions host->pool, then merges and weight changes from threads
    struct J { std::vector<ft_desc> d; std::vector<uint32_t> w; std::vector<ft_off_t> offs; ft_job_t id = 0; bool merged = false; };
    auto make = [&](uint32_t nfunc, uint64_t lo, uint64_t hi, bool p2p) {
      J j;
      for (uint32_t f = 0; f < nfunc; ++f) {
        const uint64_t n = lo + r() % (hi - lo + 1);
        ft_off_t off = 0;
        OK(ft_slab_alloc(pool, n + 32, &off));
        ft_desc d{};
        d.func = f; d.dst_space = FT_POOL; d.dst = off + r() % 16; d.row_bytes = n; d.rows = 1; d.src_pitch = d.dst_pitch = n;
        if (p2p) {
          ft_off_t s = 0;
          OK(ft_slab_alloc(pool, n + 32, &s));
          const uint64_t so = s + r() % 16, ho = r() % (host_bytes / 2 - n);
          HIPOK(hipMemcpy(dev + so, host + ho, n, hipMemcpyHostToDevice));
          std::memcpy(expect.data() + so, host + ho, n);
          d.src_space = FT_POOL; d.src = so;
          std::memcpy(expect.data() + d.dst, host + ho, n);
          j.offs.push_back(s);
        } else {
          const uint64_t ho = r() % (host_bytes / 2 - n);
          d.src_space = FT_HOST; d.src = reinterpret_cast<uint64_t>(host + ho);
          std::memcpy(expect.data() + d.dst, host + ho, n);
        }
        j.offs.push_back(off);
        j.d.push_back(d);
        j.w.push_back(1 + r() % 7);
      }
      return j;
    };
    J first = make(4, 8 * MiB, 24 * MiB, false);
    {
      J extra = make(2, 16 * MiB, 32 * MiB, true);  // pool->pool functions in the same open job
      for (auto &d : extra.d) { d.func += 4; first.d.push_back(d); }
      first.w.insert(first.w.end(), extra.w.begin(), extra.w.end());
      first.offs.insert(first.offs.end(), extra.offs.begin(), extra.offs.end());
    }
    {
      // function 6 comes from pageable memory, function 7 goes to it
      const uint64_t n = 6 * MiB + r() % MiB;
      ft_off_t in = 0, out = 0;
      OK(ft_slab_alloc(pool, n + 32, &in));
      OK(ft_slab_alloc(pool, n + 32, &out));
      first.offs.push_back(in);
      first.offs.push_back(out);
      const uint64_t from = r() % (page_bytes / 2 - n), to = page_bytes / 2 + r() % 16, fill = r() % (host_bytes / 2 - n);
      HIPOK(hipMemcpy(dev + out + 3, host + fill, n, hipMemcpyHostToDevice));
      std::memcpy(expect.data() + out + 3, host + fill, n);
      ft_desc a{}, b{};
      a.func = 6; a.src_space = FT_PAGEABLE; a.src = reinterpret_cast<uint64_t>(pageable.data() + from);
      a.dst_space = FT_POOL; a.dst = in + 7; a.row_bytes = n; a.rows = 1; a.src_pitch = a.dst_pitch = n;
      std::memcpy(expect.data() + a.dst, pageable.data() + from, n);
      b.func = 7; b.src_space = FT_POOL; b.src = out + 3;
      b.dst_space = FT_PAGEABLE; b.dst = reinterpret_cast<uint64_t>(pageable.data() + to); b.row_bytes = n; b.rows = 1; b.src_pitch = b.dst_pitch = n;
      std::memcpy(pageable_expect.data() + to, host + fill, n);
      first.d.push_back(a);
      first.d.push_back(b);
      first.w.push_back(2);
      first.w.push_back(3);
    }
    std::vector<J> later;
    for (int i = 0; i < 6; ++i) later.push_back(make(1 + i % 3, 64 * 1024, 3 * MiB, i % 2 == 1));
    OK(ft_submit_transfers(pool, first.d.data(), (uint32_t)first.d.size(), first.w.data(), (uint32_t)first.w.size(), 256 * 1024,
                           FT_OPEN | FT_KEEP, stream, &first.id));
    std::atomic<int> stop{0};
    std::thread changer([&] {
      std::mt19937_64 q(round);
      while (!stop.load()) {
        std::vector<uint32_t> w(first.w.size());
        for (auto &x : w) x = 1 + q() % 9;
        uint64_t at[3];
        int rc = ft_job_reweight(pool, first.id, w.data(), (uint32_t)w.size(), nullptr, at);
        if (rc != 0) { std::fprintf(stderr, "reweight rc %d\n", rc); std::abort(); }
        std::this_thread::sleep_for(std::chrono::microseconds(50 + q() % 200));
      }
    });
    auto merger = [&](int from) {
      hipStream_t s;
      HIPOK(hipStreamCreate(&s));
      for (int i = from; i < 6; i += 2) {
        J &j = later[i];
        int rc = ft_submit_merge(pool, first.id, j.d.data(), (uint32_t)j.d.size(), j.w.data(), (uint32_t)j.w.size(), 0, s, &j.id);
        if (rc == FT_ECLOSED) rc = ft_submit_transfers(pool, j.d.data(), (uint32_t)j.d.size(), j.w.data(), (uint32_t)j.w.size(), 256 * 1024, 0, s, &j.id);
        else j.merged = true;
        if (rc != 0) { std::fprintf(stderr, "merge rc %d\n", rc); std::abort(); }
        OK(ft_wait(pool, j.id));
        (void)ft_job_release(pool, j.id);
      }
      HIPOK(hipStreamSynchronize(s));
      HIPOK(hipStreamDestroy(s));
    };
    std::thread m0(merger, 0), m1(merger, 1);
    OK(ft_wait(pool, first.id));
    m0.join();
    m1.join();
    stop.store(1);
    changer.join();
    (void)ft_job_release(pool, first.id);
    // closed jobs: one small (tables with the launch), one larger (counter pair), one plain
    for (uint64_t n : {uint64_t(4096), 3 * MiB, 40 * MiB}) {
      J j = make(1 + (n > MiB ? 2 : 0), n, n + 100, n == 3 * MiB);
      OK(ft_submit_transfers(pool, j.d.data(), (uint32_t)j.d.size(), j.w.data(), (uint32_t)j.w.size(), 2 * MiB, round % 2 ? FT_VALIDATE : 0, stream, &j.id));
      OK(ft_wait(pool, j.id));
      (void)ft_job_release(pool, j.id);
      for (ft_off_t o : j.offs) (void)o;
      later.push_back(std::move(j));
    }
    {
      // a closed job with a little pageable memory on both sides: through a pinned buffer of its own
      const uint64_t n = 3 * MiB / 16 + r() % 1000;
      ft_off_t in = 0, out = 0;
      OK(ft_slab_alloc(pool, n + 32, &in));
      OK(ft_slab_alloc(pool, n + 32, &out));
      first.offs.push_back(in);
      first.offs.push_back(out);
      const uint64_t from = r() % (page_bytes / 2 - n), to = page_bytes / 2 + 16 * MiB + r() % 16, fill = r() % (host_bytes / 2 - n);
      HIPOK(hipMemcpy(dev + out + 1, host + fill, n, hipMemcpyHostToDevice));
      std::memcpy(expect.data() + out + 1, host + fill, n);
      ft_desc d2[2] = {};
      d2[0].func = 0; d2[0].src_space = FT_PAGEABLE; d2[0].src = reinterpret_cast<uint64_t>(pageable.data() + from);
      d2[0].dst_space = FT_POOL; d2[0].dst = in + 9; d2[0].row_bytes = n; d2[0].rows = 1;
      d2[1].func = 1; d2[1].src_space = FT_POOL; d2[1].src = out + 1;
      d2[1].dst_space = FT_PAGEABLE; d2[1].dst = reinterpret_cast<uint64_t>(pageable.data() + to); d2[1].row_bytes = n; d2[1].rows = 1;
      std::memcpy(expect.data() + in + 9, pageable.data() + from, n);
      std::memcpy(pageable_expect.data() + to, host + fill, n);
      const uint32_t w2[2] = {1, 2};
      ft_job_t id = 0;
      OK(ft_submit_transfers(pool, d2, 2, w2, 2, 2 * MiB, 0, stream, &id));
      OK(ft_wait(pool, id));
    }
    HIPOK(hipDeviceSynchronize());
    std::vector<char> got(pool_bytes);
    HIPOK(hipMemcpy(got.data(), dev, pool_bytes, hipMemcpyDeviceToHost));
    if (std::memcmp(got.data(), expect.data(), pool_bytes) != 0) { std::fprintf(stderr, "bytes differ in round %d\n", round); std::abort(); }
    if (pageable != pageable_expect) { std::fprintf(stderr, "pageable bytes differ in round %d\n", round); std::abort(); }
    for (ft_off_t o : first.offs) OK(ft_slab_free(pool, o));
    for (J &j : later) for (ft_off_t o : j.offs) OK(ft_slab_free(pool, o));
  }
  // the store on top
  {
    char *spill = host + host_bytes / 2;
    ft_store *st = nullptr;
    OK(ft_store_create(&st, pool, spill, 256 * MiB, 48 * MiB, 2 * MiB, stream));
    for (uint64_t id = 1; id <= 30; ++id) {
      ft_off_t off = 0;
      OK(ft_store_put(st, id, (1 + id % 5) * 2 * MiB, 40 - id + id % 7, &off));
      if (id % 3 == 0) { uint32_t was = 0; OK(ft_store_get(st, id - 2, &off, &was)); OK(ft_store_done(st, id - 2)); }
      OK(ft_store_advance(st, 1));
    }
    ft_store_stats_t s{};
    OK(ft_store_stats(st, &s));
    std::fprintf(stderr, "store: out %llu in %llu stalls %llu\n", (unsigned long long)s.moved_out, (unsigned long long)s.moved_in, (unsigned long long)s.stalls);
    OK(ft_store_destroy(st));
  }
  HIPOK(hipStreamSynchronize(stream));
  OK(ft_pool_destroy(pool));
  HIPOK(hipStreamDestroy(stream));
  HIPOK(hipHostFree(host));
  HIPOK(hipFree(dev));
  std::printf("c_abi_stress done\n");
  return 0;
}
