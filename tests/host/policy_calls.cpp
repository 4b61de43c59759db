// Host check of the policy and path planners (no GPU involved), built with the address and
// undefined-behaviour sanitizers: random call sequences with exactly-sized output arrays, so that a
// write or read past what the header promises is caught. Results are only checked for what the
// header states outright (counts within bounds, conservation of bandwidth, every chunk on a path);
// the values themselves are compared with the oracle by the Python tests.
// Usage: policy_calls <first seed> <count>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>
#include "../../include/faastube.h"
static uint64_t g_seed;
#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "FAIL %s line %d seed %llu\n", #c, __LINE__, (unsigned long long)g_seed); std::abort(); } } while (0)

int main(int argc, char **argv) {
  const uint64_t first = argc > 1 ? strtoull(argv[1], 0, 10) : 1, count = argc > 2 ? strtoull(argv[2], 0, 10) : 200;
  for (g_seed = first; g_seed < first + count; ++g_seed) {
    std::mt19937_64 r(g_seed);
    auto U = [&](uint64_t a, uint64_t b) { return a + r() % (b - a + 1); };
    {  // migration planner
      const uint32_t n = (uint32_t)U(0, 40);
      std::vector<ft_object> o(n);
      uint64_t resident = 0;
      for (uint32_t i = 0; i < n; ++i) {
        o[i] = ft_object{i * 3 + U(0, 2), U(1, 1000), U(0, 12), (uint32_t)U(0, 1), 0};
        if (o[i].resident) resident += o[i].bytes;
      }
      std::vector<uint64_t> ev(n), rl(n);
      uint32_t ne = 0, nr = 0;
      const uint64_t cap = U(1, 12000), inc = U(0, 1500);
      for (uint32_t pol = 0; pol < 2; ++pol) {
        int rc = ft_migrate_plan(n ? o.data() : nullptr, n, cap, inc, pol, n ? ev.data() : nullptr, &ne,
                                 n ? rl.data() : nullptr, &nr);
        if (rc != FT_OK) continue;
        CHECK(ne <= n && nr <= n);
        CHECK(!(ne > 0 && nr > 0));
        uint64_t out = 0;
        for (uint32_t i = 0; i < ne; ++i)
          for (auto &x : o) if (x.id == ev[i]) { CHECK(x.resident); out += x.bytes; }
        if (resident + inc > cap && resident - out + inc > cap) CHECK(out == resident);  // everything went and it still does not fit
      }
    }
    {  // pool sizing
      ft_sizer *s = nullptr;
      CHECK(ft_sizer_create(&s, U(0, 1000), r() % 2 ? 0.0 : 0.5 + (double)U(0, 49) / 100.0, 1.0 + (double)U(0, 50)) == FT_OK);
      double t = 0;
      for (int i = 0; i < 200; ++i) {
        t += (double)U(0, 1000) / 100.0;
        CHECK(ft_sizer_observe(s, (uint32_t)U(0, 5), t, U(0, 1u << 20), (uint32_t)U(1, 8)) == FT_OK);
        uint64_t b = 0;
        CHECK(ft_sizer_target(s, t + (double)U(0, 2000) / 100.0, &b) == FT_OK);
      }
      CHECK(ft_sizer_destroy(s) == FT_OK);
    }
    {  // path planner
      const uint32_t n = (uint32_t)U(2, 16);
      std::vector<uint32_t> topo(n * n, 0);
      const bool mesh = r() % 2;
      uint64_t total = 0;
      for (uint32_t u = 0; u < n; ++u)
        for (uint32_t v = 0; v < n; ++v)
          if (u != v && (mesh || r() % 3 == 0)) { topo[u * n + v] = (uint32_t)U(1, 4) * 24; total += topo[u * n + v]; }
      ft_links *l = nullptr;
      CHECK(ft_links_create(&l, n, topo.data(), n > 8 ? (uint32_t)U(1, 4) : (uint32_t)U(0, 4)) == FT_OK);
      std::vector<uint32_t> live;
      for (int step = 0; step < 30; ++step) {
        const uint32_t func = (uint32_t)U(0, 9);
        const uint32_t src = (uint32_t)U(0, n - 1), dst = (uint32_t)U(0, n - 1);
        int rc = ft_links_select(l, func, src, dst);
        CHECK(rc == FT_OK || rc == FT_EINVAL);
        uint32_t np = 0;
        // ask with exactly the room needed: first with none to learn the counts
        std::vector<uint32_t> nodes(16 * 64), len(64), bw(64);
        rc = ft_links_paths(l, func, nodes.data(), (uint32_t)nodes.size(), len.data(), bw.data(), 64, &np);
        if (rc == FT_OK) {
          uint32_t used = 0;
          for (uint32_t i = 0; i < np; ++i) { CHECK(len[i] >= 2 && len[i] <= n); used += len[i]; }
          std::vector<uint32_t> nodes2(used ? used : 1), len2(np ? np : 1), bw2(np ? np : 1);
          uint32_t np2 = 0;
          CHECK(ft_links_paths(l, func, nodes2.data(), used, len2.data(), bw2.data(), np, &np2) == FT_OK && np2 == np);
          if (used > 1) {
            uint32_t np3 = 0;
            CHECK(ft_links_paths(l, func, nodes2.data(), used - 1, len2.data(), bw2.data(), np, &np3) == FT_EINVAL);
          }
        }
        if (r() % 3 == 0) (void)ft_links_release(l, (uint32_t)U(0, 9));
        std::vector<uint32_t> fr(n * n);
        CHECK(ft_links_free(l, fr.data()) == FT_OK);
        for (uint32_t i = 0; i < n * n; ++i) CHECK(fr[i] <= topo[i]);
      }
      for (uint32_t f = 0; f < 10; ++f) (void)ft_links_release(l, f);
      std::vector<uint32_t> fr(n * n);
      CHECK(ft_links_free(l, fr.data()) == FT_OK);
      for (uint32_t i = 0; i < n * n; ++i) CHECK(fr[i] == topo[i]);  // all bandwidth is back
      CHECK(ft_links_destroy(l) == FT_OK);
    }
    {  // striping
      const uint32_t np = (uint32_t)U(1, 8);
      std::vector<uint32_t> bw(np);
      for (auto &b : bw) b = (uint32_t)U(1, 200);
      const uint64_t nc = U(0, 500);
      std::vector<uint32_t> path(nc ? nc : 1);
      CHECK(ft_stripe_chunks(bw.data(), np, nc, path.data()) == FT_OK);
      for (uint64_t c = 0; c < nc; ++c) CHECK(path[c] < np);
    }
  }
  std::printf("done %llu..%llu\n", (unsigned long long)first, (unsigned long long)(first + count - 1));
  return 0;
}
