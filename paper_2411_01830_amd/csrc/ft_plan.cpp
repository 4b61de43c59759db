#include "ft_plan.h"

#include <algorithm>
#include <numeric>

namespace ft {

void tile_shape(uint64_t chunk_bytes, uint64_t want_tile, uint64_t *tile_bytes, uint32_t *tiles_per_chunk) {
  if (want_tile < 16) want_tile = 16;
  uint64_t n = (chunk_bytes + want_tile - 1) / want_tile;
  if (n > 0xffffu) n = 0xffffu;
  uint64_t tile = (chunk_bytes + n - 1) / n;
  tile = (tile + 15) & ~15ull;
  *tile_bytes = tile;
  *tiles_per_chunk = (uint32_t)((chunk_bytes + tile - 1) / tile);
}

// Position of chunk j of function f in the proportional order: the chunks (g, i) with
// (i+1)/w_g < (j+1)/w_f, or equal and g < f, come before it.
static uint64_t rank_of_chunk(const std::vector<Func> &funcs, uint32_t f, uint64_t j) {
  typedef unsigned __int128 u128;
  const u128 num = (u128)(j + 1);
  const uint64_t wf = funcs[f].weight;
  uint64_t rank = j;
  for (uint32_t g = 0; g < funcs.size(); ++g) {
    if (g == f) continue;
    const u128 prod = num * funcs[g].weight;
    u128 c = prod / wf;                           // i + 1 <= prod / wf
    if (g > f && prod % wf == 0) c -= 1;          // ties go to the lower function
    rank += c < funcs[g].nchunks ? (uint64_t)c : funcs[g].nchunks;
  }
  return rank;
}

void build_chunk_table(ClassPlan &cp, uint64_t chunk_bytes, uint64_t tile_bytes, uint32_t tiles_per_chunk) {
  cp.chunk_desc.clear();
  cp.desc_per = 1;
  // A job of many small descriptors gets an entry per tile: the entry is then the tile's
  // first descriptor itself and the device searches nothing.
  if (cp.xfers.size() > 2 * cp.nchunks && cp.nchunks * tiles_per_chunk + cp.funcs.size() <= kMaxChunkTable)
    cp.desc_per = tiles_per_chunk;
  else if (cp.nchunks + cp.funcs.size() > kMaxChunkTable)
    return;
  const uint64_t step = cp.desc_per == 1 ? chunk_bytes : tile_bytes;
  cp.chunk_desc.reserve(cp.nchunks * cp.desc_per + cp.funcs.size());
  // one forward walk over each function's descriptors
  for (const Func &fn : cp.funcs) {
    const uint32_t last = fn.desc_off + fn.ndesc - 1;
    uint32_t x = fn.desc_off;
    for (uint64_t k = 0; k < fn.nchunks; ++k)
      for (uint32_t u = 0; u < cp.desc_per; ++u) {
        const uint64_t pos = (fn.chunk_base + k) * chunk_bytes + u * step;
        while (x < last && cp.xfers[x + 1].stream_off <= pos) ++x;
        cp.chunk_desc.push_back(x);
      }
    cp.chunk_desc.push_back(last);
  }
}

void build_skips(const ClassPlan &cp, uint64_t chunk_bytes, uint64_t tile_bytes, uint32_t tiles_per_chunk,
                 std::vector<Skip> *skips, uint64_t *ntickets) {
  skips->clear();
  struct Short {
    uint64_t rank, tiles;
  };
  std::vector<Short> shorts;
  for (uint32_t f = 0; f < cp.funcs.size(); ++f) {
    const Func &fn = cp.funcs[f];
    const uint64_t last_bytes = fn.stream_bytes - (fn.chunk_base + fn.nchunks - 1) * chunk_bytes;
    const uint64_t tiles = (last_bytes + tile_bytes - 1) / tile_bytes;
    if (tiles < tiles_per_chunk) shorts.push_back(Short{rank_of_chunk(cp.funcs, f, fn.nchunks - 1), tiles});
  }
  std::sort(shorts.begin(), shorts.end(), [](const Short &a, const Short &b) { return a.rank < b.rank; });
  uint64_t gone = 0;
  for (const Short &sh : shorts) {
    Skip sk;
    sk.at = sh.rank * tiles_per_chunk + sh.tiles - gone;
    sk.gap = tiles_per_chunk - sh.tiles;
    gone += sk.gap;
    skips->push_back(sk);
  }
  *ntickets = cp.nchunks * tiles_per_chunk - gone;
}

namespace {

// slot a before slot b: smaller finish tag (i+1)/w, ties to the lower function
struct SlotLess {
  const std::vector<Func> *funcs;
  bool operator()(const Slot &a, const Slot &b) const {
    uint64_t lhs = (uint64_t)(a.i + 1) * (*funcs)[b.fl].weight;
    uint64_t rhs = (uint64_t)(b.i + 1) * (*funcs)[a.fl].weight;
    if (lhs != rhs) return lhs < rhs;
    return a.fl < b.fl;
  }
};

}  // namespace

int build_phases(std::vector<Func> &funcs, std::vector<Phase> &phases, std::vector<Slot> &slots,
                 uint64_t *nchunks_out) {
  phases.clear();
  slots.clear();
  *nchunks_out = 0;
  const uint32_t F = (uint32_t)funcs.size();
  if (F == 0) return FT_OK;
  if (F == 1) {
    // one function (passing a single tensor is the commonest job there is): its chunks in stream
    // order, one slot per round - what the general construction below arrives at, without its vectors
    funcs[0].weight = 1;
    funcs[0].chunk_off = 0;
    phases.push_back(Phase{0, 0, 0, 1});
    slots.push_back(Slot{0, 0, 1, 0});
    *nchunks_out = funcs[0].nchunks;
    return FT_OK;
  }
  uint32_t g = 0;
  for (auto &f : funcs) g = std::gcd(g, f.weight);
  for (auto &f : funcs) f.weight /= g;
  {
    // only meaningful while the chunk table is built (it is not when this would wrap)
    uint64_t acc = 0;
    for (auto &f : funcs) {
      f.chunk_off = (uint32_t)acc;
      acc += f.nchunks + 1;
    }
  }

  std::vector<uint64_t> q(F), r(F);
  std::vector<char> present(F, 1);
  uint64_t W = 0;
  for (uint32_t i = 0; i < F; ++i) {
    q[i] = funcs[i].nchunks / funcs[i].weight;
    r[i] = funcs[i].nchunks % funcs[i].weight;
    W += funcs[i].weight;
  }
  // A round can hold at most min(W, N) chunks, and there are at most 2F+1 phases.
  uint64_t N = 0;
  for (auto &f : funcs) N += f.nchunks;
  if (std::min<uint64_t>(W, N) > kMaxSlots) return FT_EINVAL;

  // full round of the present set, sorted once, then only filtered
  std::vector<Slot> cur;
  bool cur_valid = false;
  auto rebuild = [&]() -> int {
    uint64_t need = 0;
    for (uint32_t i = 0; i < F; ++i)
      if (present[i]) need += funcs[i].weight;
    if (need > kMaxSlots) return FT_EINVAL;
    cur.clear();
    cur.reserve(need);
    for (uint32_t i = 0; i < F; ++i)
      if (present[i])
        for (uint32_t j = 0; j < funcs[i].weight; ++j) cur.push_back(Slot{i, j, funcs[i].weight, funcs[i].chunk_off});
    std::sort(cur.begin(), cur.end(), SlotLess{&funcs});
    cur_valid = true;
    return FT_OK;
  };

  uint64_t R = 0, rank = 0;
  uint32_t left = F;
  while (left > 0) {
    uint64_t Q = ~0ull;
    for (uint32_t i = 0; i < F; ++i)
      if (present[i]) Q = std::min(Q, q[i]);
    if (Q > R) {
      // rounds R .. Q-1: every present function fills its whole share
      if (!cur_valid) {
        int rc = rebuild();
        if (rc != FT_OK) return rc;
      }
      if (slots.size() + cur.size() > kMaxSlots) return FT_EINVAL;
      Phase ph;
      ph.rank_base = rank;
      ph.round_base = R;
      ph.slot_off = (uint32_t)slots.size();
      ph.nslots = (uint32_t)cur.size();
      slots.insert(slots.end(), cur.begin(), cur.end());
      phases.push_back(ph);
      rank += (uint64_t)ph.nslots * (Q - R);
      R = Q;
    }
    // round R: functions with q == R either are gone (r == 0) or fill r of their w slots
    bool any_partial = false;
    for (uint32_t i = 0; i < F; ++i)
      if (present[i] && q[i] == R) {
        if (r[i] == 0) {
          present[i] = 0;
          --left;
          cur_valid = false;
        } else {
          any_partial = true;
        }
      }
    if (!any_partial) continue;
    // one irregular round. When the weights dwarf the chunk counts the full round may
    // be far larger than what is left, so build from the remaining chunks directly.
    std::vector<Slot> irr;
    uint64_t need = 0;
    for (uint32_t i = 0; i < F; ++i)
      if (present[i]) need += (q[i] == R) ? r[i] : funcs[i].weight;
    if (slots.size() + need > kMaxSlots) return FT_EINVAL;
    irr.reserve(need);
    for (uint32_t i = 0; i < F; ++i)
      if (present[i]) {
        uint32_t cnt = (q[i] == R) ? (uint32_t)r[i] : funcs[i].weight;
        for (uint32_t j = 0; j < cnt; ++j) irr.push_back(Slot{i, j, funcs[i].weight, funcs[i].chunk_off});
      }
    std::sort(irr.begin(), irr.end(), SlotLess{&funcs});
    Phase ph;
    ph.rank_base = rank;
    ph.round_base = R;
    ph.slot_off = (uint32_t)slots.size();
    ph.nslots = (uint32_t)irr.size();
    slots.insert(slots.end(), irr.begin(), irr.end());
    phases.push_back(ph);
    rank += ph.nslots;
    for (uint32_t i = 0; i < F; ++i)
      if (present[i] && q[i] == R) {
        present[i] = 0;
        --left;
        cur_valid = false;
      }
    R += 1;
  }
  *nchunks_out = rank;
  return FT_OK;
}

namespace {

bool mul_overflow(uint64_t a, uint64_t b, uint64_t *out) { return __builtin_mul_overflow(a, b, out); }
bool add_overflow(uint64_t a, uint64_t b, uint64_t *out) { return __builtin_add_overflow(a, b, out); }

// bytes from the first to one past the last byte touched; false on wrap
bool extent_of(uint64_t row_bytes, uint64_t rows, uint64_t pitch, uint64_t *out) {
  uint64_t span;
  if (rows == 1) {
    *out = row_bytes;
    return true;
  }
  if (mul_overflow(rows - 1, pitch, &span)) return false;
  return !add_overflow(span, row_bytes, out);
}

struct Interval {
  uint64_t lo, hi;
};

void push_rows(std::vector<Interval> &v, uint64_t base, uint64_t row_bytes, uint64_t rows, uint64_t pitch) {
  if (rows == 1 || pitch == row_bytes) {
    v.push_back(Interval{base, base + row_bytes * rows});
    return;
  }
  for (uint64_t r = 0; r < rows; ++r) v.push_back(Interval{base + r * pitch, base + r * pitch + row_bytes});
}

bool overlaps(std::vector<Interval> &dst, std::vector<Interval> &src) {
  auto by_lo = [](const Interval &a, const Interval &b) { return a.lo < b.lo; };
  std::sort(dst.begin(), dst.end(), by_lo);
  for (size_t i = 1; i < dst.size(); ++i)
    if (dst[i].lo < dst[i - 1].hi) return true;
  // destinations are disjoint and sorted, so their ends are sorted as well
  for (const Interval &s : src) {
    auto it = std::upper_bound(dst.begin(), dst.end(), s.lo,
                               [](uint64_t v, const Interval &d) { return v < d.hi; });
    if (it != dst.end() && it->lo < s.hi) return true;
  }
  return false;
}

}  // namespace

int plan_submit(SlabPool &pool, const std::vector<HostWindow> &windows, const ft_desc *descs,
                uint32_t ndesc, const uint32_t *weights, uint32_t nfunc, uint64_t chunk_bytes,
                uint32_t flags, SubmitPlan *out) {
  out->has_pageable = false;
  // ---- pass 1: malformed arguments
  if (nfunc == 0 || weights == nullptr) return FT_EINVAL;
  if (ndesc != 0 && descs == nullptr) return FT_EINVAL;
  for (uint32_t f = 0; f < nfunc; ++f)
    if (weights[f] == 0) return FT_EINVAL;
  if (chunk_bytes == 0 || chunk_bytes % 16 != 0) return FT_EINVAL;
  for (uint32_t i = 0; i < ndesc; ++i) {
    const ft_desc &d = descs[i];
    if (d.func >= nfunc || d.flags != 0) return FT_EINVAL;
    if (d.src_space > FT_PAGEABLE || d.dst_space > FT_PAGEABLE) return FT_EINVAL;
    if (d.src_space != FT_POOL && d.dst_space != FT_POOL) return FT_EINVAL;  // host to host
    if (d.row_bytes == 0 || d.rows == 0) return FT_EINVAL;
    if (d.rows > 1 && (d.src_pitch < d.row_bytes || d.dst_pitch < d.row_bytes)) return FT_EINVAL;
  }

  // ---- pass 2: ranges; resolve both sides to device-visible addresses
  std::vector<Xfer> resolved(ndesc);
  std::vector<uint64_t> used;
  // The allocations met last, most recent first: descriptors of one submit mostly name the
  // same few (the crops of a frame, the packed buffer of a consumer), and a hit spares the
  // search of the allocation map, the search of the segment list and an entry in `used`.
  struct Recent {
    uint64_t lo = 1, hi = 0;  // offsets of the allocation, [lo, hi)
    uint64_t dev = 0;         // device address of its first byte
  };
  Recent recent[4];
  for (uint32_t i = 0; i < ndesc; ++i) {
    const ft_desc &d = descs[i];
    Xfer x;
    x.row_bytes = d.row_bytes;
    x.rows = d.rows;
    x.src_pitch = d.rows > 1 ? d.src_pitch : d.row_bytes;
    x.dst_pitch = d.rows > 1 ? d.dst_pitch : d.row_bytes;
    x.stream_off = 0;
    x.staged = (d.src_space == FT_PAGEABLE ? kStagedSrc : 0) | (d.dst_space == FT_PAGEABLE ? kStagedDst : 0);
    if (x.staged) out->has_pageable = true;
    uint64_t payload;
    if (mul_overflow(d.row_bytes, d.rows, &payload)) return FT_ERANGE;
    for (int side = 0; side < 2; ++side) {
      uint64_t off = side == 0 ? d.src : d.dst;
      uint8_t space = side == 0 ? d.src_space : d.dst_space;
      uint64_t ext, end;
      if (!extent_of(d.row_bytes, d.rows, side == 0 ? x.src_pitch : x.dst_pitch, &ext)) return FT_ERANGE;
      if (add_overflow(off, ext, &end)) return FT_ERANGE;
      uint64_t addr;
      if (space == FT_POOL) {
        int hit = -1;
        for (int k = 0; k < 4; ++k)
          if (off >= recent[k].lo && off < recent[k].hi && ext <= recent[k].hi - off) {
            hit = k;
            break;
          }
        if (hit < 0) {
          uint64_t start;
          const Allocation *al = pool.owner(off, ext, &start);
          if (al == nullptr) return FT_ERANGE;
          used.push_back(start);
          Recent r;
          r.lo = start;
          r.hi = start + al->nslabs * pool.slab_bytes();
          r.dev = reinterpret_cast<uint64_t>(pool.ptr(start));  // an allocation lies in one segment
          recent[3] = recent[2];
          recent[2] = recent[1];
          recent[1] = recent[0];
          recent[0] = r;
          hit = 0;
        }
        addr = recent[hit].dev + (off - recent[hit].lo);
      } else if (space == FT_PAGEABLE) {
        // read or written by the library's own threads: only memory the caller has vouched for
        bool inside = false;
        for (const HostWindow &w : windows)
          if (w.pageable && off >= w.base && end <= w.base + w.bytes) inside = true;
        if (!inside) return FT_ERANGE;
        addr = off;
      } else {
        bool any = false, inside = false;
        for (const HostWindow &w : windows) {
          if (w.pageable) continue;
          any = true;
          if (off >= w.base && end <= w.base + w.bytes) inside = true;
        }
        if (any ? !inside : off == 0) return FT_ERANGE;
        addr = off;
      }
      if (side == 0) x.src = addr; else x.dst = addr;
    }
    resolved[i] = x;
  }

  // ---- pass 3: exact aliasing check, on request
  if (flags & FT_VALIDATE) {
    // Rows can only collide if the spans of their descriptors' sides do (first to last byte
    // touched). The sides of one space are therefore grouped by overlapping spans first, and
    // only groups that hold a destination and at least one more side are compared row by row:
    // packed destinations and sources in other allocations, the usual case, cost a sort of
    // 2 x ndesc spans instead of a sort of every row (1536 crops: 7 ms -> 0.1 ms).
    struct Side {
      uint64_t lo, hi;
      uint32_t desc;
      bool is_dst;
    };
    for (int space = 0; space <= FT_PAGEABLE; ++space) {
      std::vector<Side> sides;
      for (uint32_t i = 0; i < ndesc; ++i) {
        const ft_desc &d = descs[i];
        const Xfer &x = resolved[i];
        uint64_t ext = 0;
        // compare in the caller's own coordinates of that space (offsets or addresses)
        if (d.dst_space == space) {
          extent_of(x.row_bytes, x.rows, x.dst_pitch, &ext);  // cannot wrap: checked in pass 2
          sides.push_back(Side{d.dst, d.dst + ext, i, true});
        }
        if (d.src_space == space) {
          extent_of(x.row_bytes, x.rows, x.src_pitch, &ext);
          sides.push_back(Side{d.src, d.src + ext, i, false});
        }
      }
      std::sort(sides.begin(), sides.end(), [](const Side &a, const Side &b) { return a.lo < b.lo; });
      std::vector<Interval> dst, src;
      size_t g0 = 0;
      while (g0 < sides.size()) {
        size_t g1 = g0 + 1;
        uint64_t reach = sides[g0].hi;
        bool has_dst = sides[g0].is_dst;
        while (g1 < sides.size() && sides[g1].lo < reach) {
          reach = std::max(reach, sides[g1].hi);
          has_dst = has_dst || sides[g1].is_dst;
          ++g1;
        }
        if (has_dst && g1 - g0 > 1)
          for (size_t k = g0; k < g1; ++k) {
            const Xfer &x = resolved[sides[k].desc];
            if (sides[k].is_dst) push_rows(dst, sides[k].lo, x.row_bytes, x.rows, x.dst_pitch);
            else push_rows(src, sides[k].lo, x.row_bytes, x.rows, x.src_pitch);
          }
        g0 = g1;
      }
      if (overlaps(dst, src)) return FT_EOVERLAP;
    }
  }

  // ---- split by class, per-function streams in submission order
  std::sort(used.begin(), used.end());
  used.erase(std::unique(used.begin(), used.end()), used.end());
  out->allocs = used;
  for (int c = 0; c < FT_NCLASS; ++c) {
    ClassPlan &cp = out->cls[c];
    cp = ClassPlan();
    auto class_of = [](const ft_desc &d) {
      return d.src_space != FT_POOL ? FT_H2P : (d.dst_space != FT_POOL ? FT_P2H : FT_P2P);
    };
    bool any = false;
    for (uint32_t i = 0; i < ndesc && !any; ++i) any = class_of(descs[i]) == c;
    if (!any) continue;  // a class without traffic costs no allocation (passing one tensor: two of three)
    if (ndesc == 1) {
      // one descriptor: one function with one stream, nothing to count or to sort into place
      Xfer x = resolved[0];
      if (x.rows > 1 && x.src_pitch == x.row_bytes && x.dst_pitch == x.row_bytes) {
        x.row_bytes *= x.rows;  // rows that touch are one contiguous run (cannot wrap: checked in pass 2)
        x.rows = 1;
        x.src_pitch = x.dst_pitch = x.row_bytes;
      }
      x.stream_off = 0;
      Func fn;
      fn.stream_bytes = x.row_bytes * x.rows;
      fn.nchunks = fn.stream_bytes / chunk_bytes + (fn.stream_bytes % chunk_bytes != 0);
      fn.func = descs[0].func;
      fn.weight = weights[descs[0].func];
      fn.desc_off = 0;
      fn.ndesc = 1;
      fn.chunk_off = 0;
      fn._pad = 0;
      fn.chunk_base = 0;
      cp.funcs.push_back(fn);
      cp.xfers.push_back(x);
      cp.payload = fn.stream_bytes;
      int rc = build_phases(cp.funcs, cp.phases, cp.slots, &cp.nchunks);
      if (rc != FT_OK) return rc;
      continue;
    }
    std::vector<uint64_t> stream(nfunc, 0);
    std::vector<uint32_t> count(nfunc, 0);
    for (uint32_t i = 0; i < ndesc; ++i)
      if (class_of(descs[i]) == c) {
        count[descs[i].func] += 1;
        uint64_t pay = resolved[i].row_bytes * resolved[i].rows;
        if (add_overflow(stream[descs[i].func], pay, &stream[descs[i].func])) return FT_ERANGE;
      }
    std::vector<int64_t> slot_of(nfunc, -1);
    uint32_t off = 0;
    for (uint32_t f = 0; f < nfunc; ++f) {
      if (stream[f] == 0) continue;
      Func fn;
      fn.stream_bytes = stream[f];
      fn.nchunks = stream[f] / chunk_bytes + (stream[f] % chunk_bytes != 0);
      fn.func = f;
      fn.weight = weights[f];
      fn.desc_off = off;
      fn.ndesc = count[f];
      fn.chunk_off = 0;
      fn._pad = 0;
      fn.chunk_base = 0;
      off += count[f];
      slot_of[f] = (int64_t)cp.funcs.size();
      cp.funcs.push_back(fn);
      cp.payload += stream[f];
    }
    cp.xfers.resize(off);
    std::vector<uint32_t> fill(cp.funcs.size(), 0);
    std::vector<uint64_t> run(cp.funcs.size(), 0);
    for (uint32_t i = 0; i < ndesc; ++i)
      if (class_of(descs[i]) == c) {
        size_t fl = (size_t)slot_of[descs[i].func];
        Xfer x = resolved[i];
        // a pitched descriptor whose rows touch is one contiguous run
        if (x.rows > 1 && x.src_pitch == x.row_bytes && x.dst_pitch == x.row_bytes) {
          x.row_bytes *= x.rows;
          x.rows = 1;
          x.src_pitch = x.dst_pitch = x.row_bytes;
        }
        x.stream_off = run[fl];
        run[fl] += x.row_bytes * x.rows;
        cp.xfers[cp.funcs[fl].desc_off + fill[fl]++] = x;
      }
    int rc = build_phases(cp.funcs, cp.phases, cp.slots, &cp.nchunks);
    if (rc != FT_OK) return rc;
  }
  return FT_OK;
}

}  // namespace ft
