// Host check of the planner's tables, built with the address and undefined-behaviour sanitizers:
// random submits are planned, then every ticket is walked the way the copy kernel walks it (cursor
// over the runs of empty tiles and over the phases, slot, chunk table, descriptor search, pieces)
// with every table read checked against the table's size. Tickets must name non-empty tiles only,
// a function's tiles must come in stream order, and the pieces must add up to each function's stream.
// Usage: walk_tables <first seed> <count>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>
#include "../../paper_2411_01830_amd/csrc/ft_plan.h"
using namespace ft;
#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "FAIL %s line %d seed %llu\n", #c, __LINE__, (unsigned long long)g_seed); std::abort(); } } while (0)
static uint64_t g_seed;
static uint64_t n_planted = 0, n_per = 0, n_notable = 0, n_skips = 0, n_cls = 0, n_tickets = 0;
template <class T> const T &at(const std::vector<T> &v, uint64_t i, int line) {
  if (i >= v.size()) { std::fprintf(stderr, "OOB read line %d idx %llu size %zu seed %llu\n", line, (unsigned long long)i, v.size(), (unsigned long long)g_seed); std::abort(); }
  return v[i];
}
#define AT(v, i) at(v, i, __LINE__)

static void walk(const ClassPlan &cp, uint64_t C, uint64_t tile, uint32_t tpc, const std::vector<Skip> &skips, uint64_t ntickets) {
  uint32_t sidx = 0; uint64_t acc = 0; uint64_t next_at = skips.empty() ? ~0ull : skips[0].at;
  uint32_t pidx = 0;
  std::vector<uint64_t> moved(cp.funcs.size(), 0);
  std::vector<uint64_t> next_byte(cp.funcs.size(), 0);
  for (uint64_t t = 0; t < ntickets; ++t) {
    while (t >= next_at) { acc += AT(skips, sidx).gap; sidx++; next_at = sidx < skips.size() ? skips[sidx].at : ~0ull; }
    const uint64_t v = t + acc;
    CHECK(v == ticket_to_tile(skips.data(), (uint32_t)skips.size(), t));
    const uint64_t rank = v / tpc, ti = v % tpc;
    CHECK(rank < cp.nchunks);
    while (pidx + 1 < cp.phases.size() && rank >= cp.phases[pidx + 1].rank_base) pidx++;
    const Phase &ph = AT(cp.phases, pidx);
    const uint64_t rel = rank - ph.rank_base, round = rel / ph.nslots;
    const uint32_t s = ph.slot_off + (uint32_t)(rel - round * ph.nslots);
    const Slot &sl = AT(cp.slots, s);
    const uint32_t fl = sl.fl;
    const Func &f = AT(cp.funcs, fl);
    CHECK(sl.weight == f.weight && sl.chunk_off == f.chunk_off);
    const uint64_t k = (ph.round_base + round) * (uint64_t)sl.weight + sl.i;
    const ChunkId id = decode_rank(cp.phases.data(), (uint32_t)cp.phases.size(), cp.slots.data(), rank);
    CHECK(id.fl == fl && id.k == k);
    CHECK(k < f.nchunks);
    uint32_t x0, x1;
    if (!cp.chunk_desc.empty()) {
      const uint64_t per = cp.desc_per;
      const uint64_t e = ((uint64_t)sl.chunk_off - fl + k) * per + fl + (per > 1 ? ti : 0);
      x0 = AT(cp.chunk_desc, e);
      x1 = per > 1 ? x0 : AT(cp.chunk_desc, e + 1);
    } else {
      x0 = f.desc_off; x1 = x0 + f.ndesc - 1;
    }
    CHECK(x0 >= f.desc_off && x1 < f.desc_off + f.ndesc && x0 <= x1);
    const uint64_t c0 = (f.chunk_base + k) * C;
    uint64_t lo = ti * tile, hi = lo + tile; if (hi > C) hi = C;
    uint64_t b0 = c0 + lo, b1 = c0 + hi; if (b1 > f.stream_bytes) b1 = f.stream_bytes;
    CHECK(b0 < b1);   // tickets name only tiles that hold bytes
    CHECK(b0 == next_byte[fl]);  // a function's tiles come in stream order
    next_byte[fl] = b1;
    uint32_t x = x0 == x1 ? x0 : find_xfer(cp.xfers.data(), x0, x1, b0);
    // piece walk
    for (uint64_t b = b0; b < b1; ++x) {
      CHECK(x < f.desc_off + f.ndesc);
      const Xfer &X = AT(cp.xfers, x);
      CHECK(X.stream_off <= b && b < X.stream_off + X.row_bytes * X.rows);
      uint64_t take = X.stream_off + X.row_bytes * X.rows - b; if (take > b1 - b) take = b1 - b;
      b += take; moved[fl] += take;
    }
  }
  uint64_t total = 0;
  for (size_t i = 0; i < cp.funcs.size(); ++i) { CHECK(moved[i] == cp.funcs[i].stream_bytes); total += moved[i]; }
  CHECK(total == cp.payload);
}

int main(int argc, char **argv) {
  const uint64_t first = argc > 1 ? strtoull(argv[1], 0, 10) : 1, count = argc > 2 ? strtoull(argv[2], 0, 10) : 200;
  for (g_seed = first; g_seed < first + count; ++g_seed) {
    std::mt19937_64 r(g_seed);
    auto U = [&](uint64_t a, uint64_t b) { return a + r() % (b - a + 1); };
    const uint64_t slab = 4096ull << U(0, 4);
    SlabPool pool(slab);
    char *base = reinterpret_cast<char *>(0x7f0000000000ull);
    const uint64_t pool_bytes = 256ull << 20;
    CHECK(pool.add_segment(base, pool_bytes) == FT_OK);
    std::vector<HostWindow> win;
    const uint64_t hbase = 0x100000000ull, hbytes = 64ull << 20;
    win.push_back(HostWindow{hbase, hbytes, false});
    const uint32_t nfunc = (uint32_t)U(1, 6);
    std::vector<uint32_t> w(nfunc);
    for (auto &x : w) x = (uint32_t)(r() % 4 == 0 ? U(1, 1000) : U(1, 5));
    const uint32_t ndesc = (uint32_t)(r() % 3 == 0 ? U(1, 400) : U(1, 12));
    std::vector<ft_desc> d(ndesc);
    uint64_t hdst = 32ull << 20;
    bool ok = true;
    for (auto &x : d) {
      x = ft_desc{};
      x.func = (uint32_t)U(0, nfunc - 1);
      x.rows = r() % 3 == 0 ? U(2, 40) : 1;
      x.row_bytes = x.rows > 1 ? U(1, 3000) : (r() % 4 == 0 ? U(1, 3u << 20) : U(1, 70000));
      x.src_pitch = x.row_bytes + (r() % 2 ? U(0, 64) : 0);
      x.dst_pitch = x.row_bytes + (r() % 2 ? U(0, 64) : 0);
      const uint64_t es = (x.rows - 1) * x.src_pitch + x.row_bytes, ed = (x.rows - 1) * x.dst_pitch + x.row_bytes;
      const int kind = (int)U(0, 2);
      uint64_t a = 0, b = 0;
      if (kind != 0 && pool.alloc(es + 16, &a) != FT_OK) { ok = false; break; }
      if (kind != 1 && pool.alloc(ed + 16, &b) != FT_OK) { ok = false; break; }
      if (kind == 0) { x.src_space = FT_HOST; x.src = hbase + U(0, (16ull << 20)); x.dst_space = FT_POOL; x.dst = b + U(0, 15); }
      else if (kind == 1) { x.src_space = FT_POOL; x.src = a + U(0, 15); x.dst_space = FT_HOST; x.dst = hbase + hdst + U(0, 15); hdst += (ed + 31) / 16 * 16; if (hdst > (60ull << 20)) { ok = false; break; } }
      else { x.src_space = FT_POOL; x.src = a + U(0, 15); x.dst_space = FT_POOL; x.dst = b + U(0, 15); }
    }
    if (!ok) continue;
    // two descriptors whose rows interleave in one allocation: their spans overlap, their rows do not
    if (r() % 3 == 0) {
      const uint64_t rb = U(1, 200), rows = U(2, 30);
      uint64_t a = 0, b = 0;
      if (pool.alloc(2 * rb * rows + 16, &a) == FT_OK && pool.alloc(2 * rb * rows + 16, &b) == FT_OK) {
        for (int half = 0; half < 2; ++half) {
          ft_desc x{};
          x.func = (uint32_t)U(0, nfunc - 1);
          x.src_space = x.dst_space = FT_POOL;
          x.rows = rows; x.row_bytes = rb; x.src_pitch = x.dst_pitch = 2 * rb;
          x.src = a + half * rb; x.dst = b + half * rb;
          d.push_back(x);
        }
      }
    }
    // a planted collision: the new destination lands inside an earlier destination's first row,
    // or the new source reads an earlier destination
    int planted = 0;
    if (r() % 4 == 0) {
      const ft_desc &victim = d[U(0, d.size() - 1)];
      if (victim.dst_space == FT_POOL) {
        ft_desc x{};
        x.func = (uint32_t)U(0, nfunc - 1);
        x.rows = 1; x.row_bytes = U(1, 64); x.src_pitch = x.dst_pitch = x.row_bytes;
        uint64_t a = 0;
        if (pool.alloc(x.row_bytes + 16, &a) == FT_OK) {
          x.src_space = x.dst_space = FT_POOL;
          const uint64_t inside = victim.dst + U(0, victim.row_bytes - 1);
          if (r() % 2) { x.src = a; x.dst = inside; x.row_bytes = x.src_pitch = x.dst_pitch = 1; planted = 1; }
          else { x.src = inside; x.dst = a; x.row_bytes = x.src_pitch = x.dst_pitch = 1; planted = 2; }
          d.push_back(x);
        }
      }
    }
    const uint32_t ndesc_all = (uint32_t)d.size();
    const uint64_t Cs[] = {16, 48, 4096, 65536, 100000 / 16 * 16, 1u << 20, 2u << 20};
    const uint64_t C = Cs[U(0, 6)];
    SubmitPlan plan;
    const bool validate = r() % 2;
    int rc = plan_submit(pool, win, d.data(), ndesc_all, w.data(), nfunc, C, validate ? FT_VALIDATE : 0, &plan);
    if (planted && validate) {
      CHECK(rc == FT_EOVERLAP);   // found, wherever it hides among the other descriptors
      n_planted++;
      continue;
    }
    CHECK(rc == FT_OK);           // nothing else collides: no false alarm either
    if (planted) continue;        // (unchecked and colliding: the order of the bytes is not defined)
    for (int c = 0; c < FT_NCLASS; ++c) {
      ClassPlan &cp = plan.cls[c];
      if (cp.nchunks == 0) continue;
      if (cp.nchunks * 8 > 4000000) continue;   // keep a case short
      const uint64_t wants[] = {16, 64, 4096, 16384, 65536, 65520, 1u << 20, 4u << 20};
      uint64_t tile; uint32_t tpc;
      tile_shape(C, wants[U(0, 7)], &tile, &tpc);
      CHECK(tile % 16 == 0 && tile > 0 && (uint64_t)tpc * tile >= C && (uint64_t)(tpc - 1) * tile < C);
      build_chunk_table(cp, C, tile, tpc);
      std::vector<Skip> skips; uint64_t nt = 0;
      build_skips(cp, C, tile, tpc, &skips, &nt);
      n_cls++; n_per += cp.desc_per > 1; n_notable += cp.chunk_desc.empty(); n_skips += !skips.empty(); n_tickets += nt;
      walk(cp, C, tile, tpc, skips, nt);
    }
  }
  std::printf("planted collisions found %llu; classes %llu, table per tile %llu, no table %llu, with skips %llu, tickets %llu\n", (unsigned long long)n_planted, (unsigned long long)n_cls, (unsigned long long)n_per, (unsigned long long)n_notable, (unsigned long long)n_skips, (unsigned long long)n_tickets);
  std::printf("done %llu..%llu\n", (unsigned long long)first, (unsigned long long)(first + count - 1));
  return 0;
}
