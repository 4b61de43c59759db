// Contention-aware selection of parallel paths between two GPUs (Sec. 6.2, Alg. 1) and the
// striping of chunks over them, host only. With one GPU per process nothing here moves
// data: it is the planner a multi-GPU engine would ask, paths in place of functions in
// the weighted chunk order.
#include <algorithm>
#include <cstdint>
#include <map>
#include <vector>

#include "../../include/faastube.h"
#include "ft_guard.h"

namespace {

typedef std::vector<uint8_t> Path;

struct Held {
  Path nodes;
  uint32_t bw;
};

}  // namespace

struct ft_links {
  uint32_t n = 0, max_hops = 0;
  std::vector<uint32_t> topo, free_bw;
  std::map<uint32_t, std::vector<Held>> paths;                  // function -> its paths
  std::map<uint32_t, std::vector<Path>> cache;                  // s * n + d -> candidate paths in order

  uint32_t &fr(uint32_t u, uint32_t v) { return free_bw[u * n + v]; }
  uint32_t tp(uint32_t u, uint32_t v) const { return topo[u * n + v]; }

  // loop-free paths s -> d of at most max_hops links, fewer hops first, then by node sequence
  const std::vector<Path> &candidates(uint32_t s, uint32_t d) {
    auto it = cache.find(s * n + d);
    if (it != cache.end()) return it->second;
    std::vector<Path> out;
    Path cur;
    cur.push_back((uint8_t)s);
    std::vector<char> seen(n, 0);
    seen[s] = 1;
    walk(cur, seen, d, out);
    std::sort(out.begin(), out.end(), [](const Path &a, const Path &b) {
      return a.size() != b.size() ? a.size() < b.size() : a < b;
    });
    return cache[s * n + d] = std::move(out);
  }
  void walk(Path &cur, std::vector<char> &seen, uint32_t d, std::vector<Path> &out) {
    const uint32_t u = cur.back();
    if (u == d) {
      out.push_back(cur);
      return;
    }
    if (cur.size() > max_hops) return;
    for (uint32_t v = 0; v < n; ++v) {
      if (tp(u, v) == 0 || seen[v]) continue;
      seen[v] = 1;
      cur.push_back((uint8_t)v);
      walk(cur, seen, d, out);
      cur.pop_back();
      seen[v] = 0;
    }
  }
  bool idle(const Path &p) {
    for (size_t i = 0; i + 1 < p.size(); ++i)
      if (fr(p[i], p[i + 1]) != tp(p[i], p[i + 1])) return false;
    return true;
  }
  uint32_t narrowest(const Path &p) const {
    uint32_t b = ~0u;
    for (size_t i = 0; i + 1 < p.size(); ++i) b = std::min(b, tp(p[i], p[i + 1]));
    return b;
  }
  void charge(const Path &p, uint32_t bw, bool take) {
    for (size_t i = 0; i + 1 < p.size(); ++i) {
      if (take) fr(p[i], p[i + 1]) -= bw; else fr(p[i], p[i + 1]) += bw;
    }
  }
  uint64_t out_free(uint32_t g) {
    uint64_t s = 0;
    for (uint32_t v = 0; v < n; ++v) s += fr(g, v);
    return s;
  }
  uint64_t in_free(uint32_t g) {
    uint64_t s = 0;
    for (uint32_t u = 0; u < n; ++u) s += fr(u, g);
    return s;
  }
  uint64_t total(uint32_t func) {
    uint64_t s = 0;
    auto it = paths.find(func);
    if (it != paths.end())
      for (const Held &h : it->second) s += h.bw;
    return s;
  }
  static bool share_link(const Path &a, const Path &b) {
    for (size_t i = 0; i + 1 < a.size(); ++i)
      for (size_t j = 0; j + 1 < b.size(); ++j)
        if (a[i] == b[j] && a[i + 1] == b[j + 1]) return true;
    return false;
  }
};

extern "C" {

int ft_links_create(ft_links **out, uint32_t n, const uint32_t *topo, uint32_t max_hops) try {
  if (out == nullptr || topo == nullptr || n < 2 || n > 16) return FT_EINVAL;
  if (max_hops == 0) max_hops = n - 1;
  if (n > 8 && max_hops > 4) return FT_EINVAL;  // keeps the number of candidate paths small
  for (uint32_t i = 0; i < n; ++i)
    if (topo[i * n + i] != 0) return FT_EINVAL;
  ft_links *l = new ft_links();
  l->n = n;
  l->max_hops = max_hops;
  l->topo.assign(topo, topo + n * n);
  l->free_bw = l->topo;
  *out = l;
  return FT_OK;
}
FT_CATCH_ALL

int ft_links_destroy(ft_links *l) {
  if (l == nullptr) return FT_EINVAL;
  delete l;
  return FT_OK;
}

int ft_links_release(ft_links *l, uint32_t func) {
  if (l == nullptr) return FT_EINVAL;
  auto it = l->paths.find(func);
  if (it == l->paths.end()) return FT_EINVAL;
  for (const Held &h : it->second) l->charge(h.nodes, h.bw, false);
  l->paths.erase(it);
  return FT_OK;
}

int ft_links_free(ft_links *l, uint32_t *free_out) {
  if (l == nullptr || free_out == nullptr) return FT_EINVAL;
  std::copy(l->free_bw.begin(), l->free_bw.end(), free_out);
  return FT_OK;
}

int ft_links_paths(ft_links *l, uint32_t func, uint32_t *nodes_out, uint32_t cap_nodes, uint32_t *len_out,
                   uint32_t *bw_out, uint32_t cap_paths, uint32_t *npaths_out) try {
  if (l == nullptr || npaths_out == nullptr) return FT_EINVAL;
  auto it = l->paths.find(func);
  if (it == l->paths.end()) return FT_EINVAL;
  *npaths_out = (uint32_t)it->second.size();
  uint32_t at = 0;
  for (uint32_t i = 0; i < it->second.size() && i < cap_paths; ++i) {
    const Held &h = it->second[i];
    if (nodes_out == nullptr || len_out == nullptr || bw_out == nullptr || at + h.nodes.size() > cap_nodes)
      return FT_EINVAL;
    for (uint8_t v : h.nodes) nodes_out[at++] = v;
    len_out[i] = (uint32_t)h.nodes.size();
    bw_out[i] = h.bw;
  }
  return FT_OK;
}
FT_CATCH_ALL

int ft_links_select(ft_links *l, uint32_t func, uint32_t src, uint32_t dst) try {
  if (l == nullptr || src >= l->n || dst >= l->n || src == dst) return FT_EINVAL;
  if (l->paths.count(func)) return FT_EINVAL;
  std::vector<Held> &mine = l->paths[func];
  const std::vector<Path> &cand = l->candidates(src, dst);  // std::map: stays valid when the cache grows
  auto saturated = [&] { return l->out_free(src) == 0 || l->in_free(dst) == 0; };
  // step 1: idle paths, shortest first
  for (const Path &p : cand) {
    if (saturated()) break;
    if (!l->idle(p)) continue;
    const uint32_t bw = l->narrowest(p);
    l->charge(p, bw, true);
    mine.push_back(Held{p, bw});
  }
  // step 2: a busy path whose one occupant holds more and can move elsewhere
  if (!saturated()) {
    for (const Path &p : cand) {
      if (saturated()) break;
      if (l->idle(p)) continue;
      bool own = false;
      for (const Held &h : mine) own = own || h.nodes == p || ft_links::share_link(p, h.nodes);
      if (own) continue;
      uint32_t blockers = 0, who = 0, which = 0;
      for (auto &kv : l->paths) {
        if (kv.first == func) continue;
        for (uint32_t i = 0; i < kv.second.size(); ++i)
          if (ft_links::share_link(p, kv.second[i].nodes)) {
            blockers += 1;
            who = kv.first;
            which = i;
          }
      }
      if (blockers != 1 || l->total(who) <= l->total(func)) continue;
      std::vector<Held> &theirs = l->paths[who];
      const Held old = theirs[which];
      l->charge(old.nodes, old.bw, false);
      const Path *alt = nullptr;
      const std::vector<Path> &other = l->candidates(old.nodes.front(), old.nodes.back());
      for (const Path &q : other)
        if (q != old.nodes && l->idle(q) && !ft_links::share_link(p, q)) {
          alt = &q;
          break;
        }
      if (alt == nullptr || !l->idle(p)) {
        l->charge(old.nodes, old.bw, true);  // back where it was
        continue;
      }
      const uint32_t abw = l->narrowest(*alt);
      l->charge(*alt, abw, true);
      theirs[which] = Held{*alt, abw};
      const uint32_t bw = l->narrowest(p);
      l->charge(p, bw, true);
      l->paths[func].push_back(Held{p, bw});
    }
  }
  return FT_OK;
}
FT_CATCH_ALL

int ft_stripe_chunks(const uint32_t *path_bw, uint32_t npaths, uint64_t nchunks, uint32_t *path_of_chunk) try {
  if (path_bw == nullptr || npaths == 0 || (nchunks != 0 && path_of_chunk == nullptr)) return FT_EINVAL;
  for (uint32_t p = 0; p < npaths; ++p)
    if (path_bw[p] == 0) return FT_EINVAL;
  std::vector<uint64_t> sent(npaths, 0);
  for (uint64_t c = 0; c < nchunks; ++c) {
    uint32_t best = 0;
    for (uint32_t p = 1; p < npaths; ++p) {
      // (sent_p + 1) / bw_p < (sent_best + 1) / bw_best, cross-multiplied
      const unsigned __int128 a = (unsigned __int128)(sent[p] + 1) * path_bw[best];
      const unsigned __int128 b = (unsigned __int128)(sent[best] + 1) * path_bw[p];
      if (a < b) best = p;
    }
    path_of_chunk[c] = best;
    sent[best] += 1;
  }
  return FT_OK;
}
FT_CATCH_ALL

}  // extern "C"
