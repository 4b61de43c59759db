// Elastic data store policies of Sec. 7, host only: the histogram rule that sizes the
// pool (Sec. 7.1) and the queue-aware choice of what to move to host memory and back
// (Sec. 7.2). No device calls; ft_pool_grow / ft_pool_shrink and the transfer engine carry
// the decisions out.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <unordered_map>
#include <vector>

#include "../../include/faastube.h"
#include "ft_guard.h"

namespace {

// nearest rank: the ceil(q*n)-th smallest
template <class T>
T percentile(std::vector<T> v, double q) {
  std::sort(v.begin(), v.end());
  double r = std::ceil(q * (double)v.size());
  size_t rank = r < 1.0 ? 1 : (r > (double)v.size() ? v.size() : (size_t)r);
  return v[rank - 1];
}

struct FuncHist {
  bool seen = false;
  double last = 0;
  std::vector<double> intervals;
  std::vector<uint64_t> sizes;
  std::vector<uint64_t> cons;
  uint64_t reserved = 0;
  double expires = 0;
};

}  // namespace

struct ft_sizer {
  uint64_t min_bytes;
  double q;
  double default_window;
  std::unordered_map<uint32_t, FuncHist> funcs;
};

extern "C" {

int ft_sizer_create(ft_sizer **out, uint64_t min_bytes, double quantile, double default_window) try {
  if (out == nullptr || quantile < 0.0 || quantile > 1.0 || !(default_window >= 0.0)) return FT_EINVAL;
  ft_sizer *s = new ft_sizer();
  s->min_bytes = min_bytes;
  s->q = quantile == 0.0 ? 0.99 : quantile;
  s->default_window = default_window;
  *out = s;
  return FT_OK;
}
FT_CATCH_ALL

int ft_sizer_destroy(ft_sizer *s) {
  if (s == nullptr) return FT_EINVAL;
  delete s;
  return FT_OK;
}

int ft_sizer_observe(ft_sizer *s, uint32_t func, double t, uint64_t data_size, uint32_t concurrency) try {
  if (s == nullptr) return FT_EINVAL;
  FuncHist &h = s->funcs[func];
  if (h.seen) h.intervals.push_back(t - h.last);
  h.seen = true;
  h.last = t;
  h.sizes.push_back(data_size);
  h.cons.push_back(concurrency);
  const uint64_t r_size = percentile(h.sizes, s->q);
  const uint64_t r_con = percentile(h.cons, s->q);
  const double r_window = h.intervals.empty() ? s->default_window : percentile(h.intervals, s->q);
  h.reserved = r_size * r_con;
  h.expires = t + r_window;
  return FT_OK;
}
FT_CATCH_ALL

int ft_sizer_target(ft_sizer *s, double t, uint64_t *bytes_out) {
  if (s == nullptr || bytes_out == nullptr) return FT_EINVAL;
  uint64_t total = 0;
  for (const auto &kv : s->funcs)
    if (kv.second.seen && t <= kv.second.expires) total += kv.second.reserved;
  *bytes_out = total > s->min_bytes ? total : s->min_bytes;
  return FT_OK;
}

int ft_migrate_plan(const ft_object *objs, uint32_t n, uint64_t capacity, uint64_t incoming, uint32_t policy,
                    uint64_t *evict_ids, uint32_t *n_evict, uint64_t *reload_ids, uint32_t *n_reload) try {
  if ((n != 0 && objs == nullptr) || n_evict == nullptr || n_reload == nullptr) return FT_EINVAL;
  if (policy != FT_EVICT_QUEUE_AWARE && policy != FT_EVICT_LRU) return FT_EINVAL;
  if (n != 0 && (evict_ids == nullptr || reload_ids == nullptr)) return FT_EINVAL;
  uint64_t used = incoming;
  std::vector<const ft_object *> in, out;
  for (uint32_t i = 0; i < n; ++i) {
    if (objs[i].resident) {
      used += objs[i].bytes;
      in.push_back(&objs[i]);
    } else {
      out.push_back(&objs[i]);
    }
  }
  if (policy == FT_EVICT_QUEUE_AWARE) {
    // furthest consumer first; of two equally far, the one stored later
    std::sort(in.begin(), in.end(), [](const ft_object *a, const ft_object *b) {
      return a->queue_pos != b->queue_pos ? a->queue_pos > b->queue_pos : a->id > b->id;
    });
  } else {
    std::sort(in.begin(), in.end(), [](const ft_object *a, const ft_object *b) { return a->id < b->id; });
  }
  uint32_t ne = 0, nr = 0;
  for (const ft_object *o : in) {
    if (used <= capacity) break;
    evict_ids[ne++] = o->id;
    used -= o->bytes;
  }
  if (ne == 0 && policy == FT_EVICT_QUEUE_AWARE) {
    // room to spare: bring back what was moved out, nearest consumer first
    std::sort(out.begin(), out.end(), [](const ft_object *a, const ft_object *b) {
      return a->queue_pos != b->queue_pos ? a->queue_pos < b->queue_pos : a->id < b->id;
    });
    for (const ft_object *o : out) {
      if (used + o->bytes > capacity) break;
      reload_ids[nr++] = o->id;
      used += o->bytes;
    }
  }
  *n_evict = ne;
  *n_reload = nr;
  return FT_OK;
}
FT_CATCH_ALL

}  // extern "C"
