// Store of intermediate results with queue-aware migration (Sec. 7.2).
//
// Results wait in the pool between the function that produced them and the function that
// will consume them. The store keeps the bytes it holds there under a budget: when a new
// result would pass it, results are moved out to host memory, the one whose consumer is
// furthest back in the request queue first (of two equally far, the one stored later);
// when a result's consumer runs and the result is out, it is brought back first (a stall);
// when room appears, results come back before they are asked for, nearest consumer first.
// Every move is an ordinary pool->host or host->pool transfer of the engine plus
// slab_alloc / slab_free on the pool and on a slab allocator over the spill arena.
#include <map>
#include <mutex>
#include <vector>

#include "../../include/faastube.h"
#include "ft_guard.h"
#include "ft_internal.h"

// Migrations run asynchronously with function execution (Sec. 7.2). A move is a job on the
// store's stream that no call of the store waits for - except ft_store_get, for the one result
// its caller is about to read. What makes that safe is the order of the work on that one stream:
// every move is an ordinary (not detached) job, so the stream passes the moves one after the
// other, and a slab or a spill slot that a move has left is handed out again at once ("in stream
// order"): whatever the caller puts there is enqueued on the store's stream after the call that
// returned it, hence after the move. A result's own move is settled (waited for, its record
// dropped) the next time the store touches that result; finished moves of other results are
// collected at the start of every call.

namespace {

struct StoreObj {
  uint64_t bytes = 0;
  uint64_t queue_pos = 0;
  bool resident = false;
  ft_off_t off = 0;     // in the pool, while resident
  uint64_t spill = 0;   // offset in the spill arena, while moved out
  ft_job_t moving = 0;  // its last move, while nobody has waited for it (0: none)
};

}  // namespace

struct ft_store {
  std::mutex mu;
  ft_pool *pool;
  char *spill_base;
  ft::SlabPool spill;
  uint64_t capacity;
  uint64_t chunk_bytes;
  void *stream;
  std::map<uint64_t, StoreObj> objs;  // by id: ids grow with store time
  ft_store_stats_t stats{};

  ft_store(ft_pool *p, char *base, uint64_t cap, uint64_t chunk, void *s)
      : pool(p), spill_base(base), spill(4096), capacity(cap), chunk_bytes(chunk), stream(s) {}
};

namespace {

// One contiguous transfer through the engine on the store's stream, not waited for.
int start_move(ft_store *s, uint8_t src_space, uint64_t src, uint8_t dst_space, uint64_t dst, uint64_t n,
               ft_job_t *job) {
  ft_desc d{};
  d.func = 0;
  d.src_space = src_space;
  d.dst_space = dst_space;
  d.src = src;
  d.dst = dst;
  d.row_bytes = n;
  d.rows = 1;
  d.src_pitch = d.dst_pitch = n;
  const uint32_t w = 1;
  return ft_submit_transfers(s->pool, &d, 1, &w, 1, s->chunk_bytes, 0, s->stream, job);
}

// Waits for the result's own move, if one is still unsettled.
int settle(ft_store *s, StoreObj &o) {
  if (o.moving == 0) return FT_OK;
  const ft_job_t job = o.moving;
  o.moving = 0;
  return ft_wait(s->pool, job);
}

// Drops the records of moves that have finished, without blocking.
void collect_finished(ft_store *s) {
  for (auto &kv : s->objs) {
    int done = 0;
    if (kv.second.moving != 0 && ft_job_done(s->pool, kv.second.moving, &done) == FT_OK && done) (void)settle(s, kv.second);
  }
}

int move_out(ft_store *s, uint64_t id) {
  StoreObj &o = s->objs[id];
  int rc = settle(s, o);  // it may just be on its way in
  if (rc != FT_OK) return rc;
  // a transfer of the caller's that has not been waited for still reads or writes the result
  // (its producer's, or a consumer that fetches it early): it cannot leave now, and stays
  if (ft::slab_busy(s->pool, o.off) != 0) return FT_EBUSY;
  uint64_t at = 0;
  rc = s->spill.alloc(o.bytes, &at);
  if (rc != FT_OK) return rc;  // FT_ENOMEM: the spill arena is full
  rc = start_move(s, FT_POOL, o.off, FT_HOST, reinterpret_cast<uint64_t>(s->spill_base + at), o.bytes, &o.moving);
  if (rc != FT_OK) {
    s->spill.free(at);
    return rc;
  }
  // the slabs go back at once: what is written there next comes after this move on the stream
  rc = ft::slab_free_ordered(s->pool, o.off);
  if (rc != FT_OK) return rc;
  o.resident = false;
  o.spill = at;
  s->stats.moved_out += 1;
  s->stats.bytes_out += o.bytes;
  s->stats.resident_bytes -= o.bytes;
  return FT_OK;
}

int move_in(ft_store *s, uint64_t id) {
  StoreObj &o = s->objs[id];
  int rc = settle(s, o);  // its move out: long over as a rule, and its record goes
  if (rc != FT_OK) return rc;
  ft_off_t off = 0;
  rc = ft_slab_alloc(s->pool, o.bytes, &off);
  if (rc != FT_OK) return rc;  // FT_ENOMEM: the pool itself is too small or too fragmented
  rc = start_move(s, FT_HOST, reinterpret_cast<uint64_t>(s->spill_base + o.spill), FT_POOL, off, o.bytes, &o.moving);
  if (rc != FT_OK) {
    (void)ft_slab_free(s->pool, off);
    return rc;
  }
  s->spill.free(o.spill);  // in stream order as well: a later move out into this slot follows this move
  o.resident = true;
  o.off = off;
  s->stats.moved_in += 1;
  s->stats.bytes_in += o.bytes;
  s->stats.resident_bytes += o.bytes;
  return FT_OK;
}

// The rule of ft_migrate_plan over the store's objects (all but `skip`), then the moves.
// reload: also bring back what fits when nothing had to go.
int make_room(ft_store *s, uint64_t incoming, const uint64_t *skip, bool reload) {
  std::vector<ft_object> view;
  for (const auto &kv : s->objs) {
    if (skip != nullptr && kv.first == *skip) continue;
    view.push_back(ft_object{kv.first, kv.second.bytes, kv.second.queue_pos, kv.second.resident ? 1u : 0u, 0});
  }
  std::vector<uint64_t> ev(view.size() + 1), rl(view.size() + 1);
  uint32_t ne = 0, nr = 0;
  int rc = ft_migrate_plan(view.data(), (uint32_t)view.size(), s->capacity, incoming, FT_EVICT_QUEUE_AWARE, ev.data(),
                           &ne, rl.data(), &nr);
  if (rc != FT_OK) return rc;
  for (uint32_t i = 0; i < ne; ++i) {
    rc = move_out(s, ev[i]);
    if (rc != FT_OK) return rc;
  }
  if (reload)
    for (uint32_t i = 0; i < nr; ++i) {
      rc = move_in(s, rl[i]);
      if (rc == FT_ENOMEM) break;  // the budget allows it, the pool does not: leave it out
      if (rc != FT_OK) return rc;
    }
  return FT_OK;
}

}  // namespace

extern "C" {

int ft_store_create(ft_store **out, ft_pool *pool, void *spill_base, uint64_t spill_bytes, uint64_t capacity,
                    uint64_t chunk_bytes, void *hip_stream) try {
  if (out == nullptr || pool == nullptr || capacity == 0) return FT_EINVAL;
  if (chunk_bytes == 0 || chunk_bytes % 16 != 0) return FT_EINVAL;
  int rc = ft::SlabPool::check_segment(spill_base, spill_bytes, 4096);
  if (rc != FT_OK) return rc;
  rc = ft_host_window_add(pool, spill_base, spill_bytes);
  if (rc != FT_OK) return rc;
  ft_store *s = new ft_store(pool, static_cast<char *>(spill_base), capacity, chunk_bytes, hip_stream);
  s->spill.add_segment(spill_base, spill_bytes);
  *out = s;
  return FT_OK;
}
FT_CATCH_ALL

int ft_store_put(ft_store *s, uint64_t id, uint64_t nbytes, uint64_t queue_pos, ft_off_t *off_out) try {
  if (s == nullptr || off_out == nullptr || nbytes == 0) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(s->mu);
  if (s->objs.count(id)) return FT_EINVAL;
  if (nbytes > s->capacity) return FT_ENOMEM;
  collect_finished(s);
  int rc = make_room(s, nbytes, nullptr, false);
  if (rc != FT_OK) return rc;
  ft_off_t off = 0;
  rc = ft_slab_alloc(s->pool, nbytes, &off);
  if (rc != FT_OK) return rc;
  StoreObj o;
  o.bytes = nbytes;
  o.queue_pos = queue_pos;
  o.resident = true;
  o.off = off;
  s->objs[id] = o;
  s->stats.resident_bytes += nbytes;
  s->stats.objects += 1;
  *off_out = off;
  return FT_OK;
}
FT_CATCH_ALL

int ft_store_get(ft_store *s, uint64_t id, ft_off_t *off_out, uint32_t *was_out) try {
  if (s == nullptr || off_out == nullptr) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(s->mu);
  auto it = s->objs.find(id);
  if (it == s->objs.end()) return FT_EINVAL;
  if (was_out) *was_out = it->second.resident ? 0u : 1u;
  collect_finished(s);
  if (!it->second.resident) {
    int rc = make_room(s, it->second.bytes, &id, false);
    if (rc != FT_OK) return rc;
    rc = move_in(s, id);
    if (rc != FT_OK) return rc;
    s->stats.stalls += 1;
  }
  // the one wait of the store: the result its caller is about to read is in place
  int rc = settle(s, it->second);
  if (rc != FT_OK) return rc;
  *off_out = it->second.off;
  return FT_OK;
}
FT_CATCH_ALL

int ft_store_done(ft_store *s, uint64_t id) try {
  if (s == nullptr) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(s->mu);
  auto it = s->objs.find(id);
  if (it == s->objs.end() || !it->second.resident) return FT_EINVAL;
  collect_finished(s);
  int rc = settle(s, it->second);
  if (rc != FT_OK) return rc;
  rc = ft_slab_free(s->pool, it->second.off);
  if (rc != FT_OK) return rc;  // FT_EBUSY: a transfer of the caller's still uses it
  s->stats.resident_bytes -= it->second.bytes;
  s->stats.objects -= 1;
  s->objs.erase(it);
  return make_room(s, 0, nullptr, true);
}
FT_CATCH_ALL

int ft_store_advance(ft_store *s, uint64_t steps) {
  if (s == nullptr) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(s->mu);
  for (auto &kv : s->objs) kv.second.queue_pos = kv.second.queue_pos > steps ? kv.second.queue_pos - steps : 0;
  return FT_OK;
}

int ft_store_sync(ft_store *s) {
  if (s == nullptr) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(s->mu);
  int rc = FT_OK;
  for (auto &kv : s->objs) {
    const int r = settle(s, kv.second);
    if (r != FT_OK) rc = r;
  }
  return rc;
}

int ft_store_stats(ft_store *s, ft_store_stats_t *out) {
  if (s == nullptr || out == nullptr) return FT_EINVAL;
  std::lock_guard<std::mutex> lock(s->mu);
  *out = s->stats;
  out->spill_used_bytes = s->spill.live_bytes();
  out->moves_in_flight = 0;
  for (const auto &kv : s->objs) out->moves_in_flight += kv.second.moving != 0 ? 1 : 0;
  return FT_OK;
}

int ft_store_destroy(ft_store *s) {
  if (s == nullptr) return FT_EINVAL;
  {
    std::lock_guard<std::mutex> lock(s->mu);
    for (auto &kv : s->objs) {
      (void)settle(s, kv.second);
      if (kv.second.resident) (void)ft_slab_free(s->pool, kv.second.off);
    }
  }
  delete s;
  return FT_OK;
}

}  // extern "C"
