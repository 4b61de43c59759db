// Open jobs: batched transfer triggering of Sec. 6.1.
//
// A chunk that has been handed to the device cannot be taken back, so a job whose whole
// order is launched at once leaves later arrivals waiting until it is done. An open job
// instead triggers its chunks in batches (5 chunks by default, as in the paper): one
// launch of the persistent copy kernel per batch, a small fixed number of batches queued
// ahead of the device, launched by a feeder thread per link class. Functions that arrive
// meanwhile (ft_submit_merge) join at the next batch that has not been triggered: the
// proportional order is built afresh over the chunks not yet triggered of every earlier
// function plus all chunks of the new ones, earlier functions first in the tie rule, and
// the following batches come from that order. Each order in force has its own tables on
// the device ("generation"); batches already queued keep the tables they were launched
// with.
//
// Circular pinned buffer of Sec. 6.1: pageable host memory (FT_PAGEABLE) cannot be read or
// written by the device. Pinning the caller's buffers per call is what the paper measures
// as too slow and caching a pinned copy of everything as too large; instead one fixed
// ring of pinned memory, (depth + 1) * batch_chunks slots of one chunk each, is shared by
// all functions: before a batch is launched the feeder and a few helper threads copy the
// stream bytes of the batch's pageable descriptors into the batch's slots (chunk i of
// batch q has slot (q mod (depth + 1)) * batch_chunks + i), the kernel reads them there,
// and the slots are used again depth + 1 batches later, when that batch is long complete.
// In the other direction (pool -> pageable host memory) the kernel writes a chunk into its
// slot and, once the batch is complete, the same threads copy it on to the destination;
// only then do the batch's chunks count as done.
#include <hip/hip_runtime_api.h>
#include <immintrin.h>

#include <algorithm>
#include <chrono>
#include <condition_variable>
#include <cstring>
#include <deque>
#include <functional>
#include <memory>
#include <mutex>
#include <thread>

#include "ft_internal.h"

namespace ft {

namespace {

struct OpenFn {
  uint64_t job;           // pool job id
  uint32_t func;          // function index inside that job
  uint32_t weight;
  uint64_t stream_bytes;
  uint64_t nchunks;       // of the whole stream
  uint64_t next_chunk;    // first chunk not yet triggered
  bool staged;            // some descriptor reads or writes pageable host memory
  uint64_t done_bytes = 0;  // bytes of its chunks whose batch has been seen complete
  std::vector<Xfer> xfers;
};

struct Generation {
  ClassPlan plan;                   // plan.funcs[i].func = index into OpenClass::fns
  std::vector<Skip> skips;
  Blob blob;
  ClassTable table{};               // device addresses; per batch: counter, range, cursors
  uint64_t ntickets = 0;
  uint64_t next_rank = 0;           // first rank of this order not yet triggered
  uint32_t next_counter = 0;
  uint32_t inflight = 0;            // batches launched with these tables and not seen complete
  hipEvent_t uploaded = nullptr;    // each of the class's two streams waits for it before its first batch
  bool waited_upload[2] = {false, false};
  // FT_LOG: one LogEntry per ticket of this order, then one WgLogEntry per workgroup of every batch
  Blob log;
  struct Triggered {
    uint64_t t0, t1;  // tickets of the batch
    uint32_t batch;   // its number in the class's sequence
  };
  std::vector<Triggered> triggered;
};

typedef HostCopy StageCopy;  // {dst, src, n}

// Copy for staging. The bytes are not touched again by this core: they go to the device or
// to a buffer that the caller reads much later, and a batch is larger than the caches. Stores
// that bypass the cache spare the read of every destination line that an ordinary store
// causes first.
__attribute__((target("avx2"))) void stream_copy_avx2(char *dst, const char *src, uint64_t n) {
  const uint64_t head = (32 - (reinterpret_cast<uintptr_t>(dst) & 31)) & 31;
  if (n < 4096 || head >= n) {
    std::memcpy(dst, src, n);
    return;
  }
  std::memcpy(dst, src, head);
  dst += head;
  src += head;
  n -= head;
  uint64_t i = 0;
  for (; i + 128 <= n; i += 128) {
    const __m256i a = _mm256_loadu_si256(reinterpret_cast<const __m256i *>(src + i));
    const __m256i b = _mm256_loadu_si256(reinterpret_cast<const __m256i *>(src + i + 32));
    const __m256i c = _mm256_loadu_si256(reinterpret_cast<const __m256i *>(src + i + 64));
    const __m256i d = _mm256_loadu_si256(reinterpret_cast<const __m256i *>(src + i + 96));
    _mm256_stream_si256(reinterpret_cast<__m256i *>(dst + i), a);
    _mm256_stream_si256(reinterpret_cast<__m256i *>(dst + i + 32), b);
    _mm256_stream_si256(reinterpret_cast<__m256i *>(dst + i + 64), c);
    _mm256_stream_si256(reinterpret_cast<__m256i *>(dst + i + 96), d);
  }
  _mm_sfence();
  std::memcpy(dst + i, src + i, n - i);
}

void stage_copy(char *dst, const char *src, uint64_t n) {
  static const bool avx2 = __builtin_cpu_supports("avx2");
  if (avx2) stream_copy_avx2(dst, src, n);
  else std::memcpy(dst, src, n);
}

struct OpenBatch {
  std::shared_ptr<Generation> gen;
  uint32_t lane = 0;                // which of the class's two streams
  hipEvent_t done = nullptr, t_begin = nullptr, t_end = nullptr;
  std::vector<std::pair<uint64_t, uint64_t>> job_chunks;  // job id, chunks of it in this batch
  std::vector<std::pair<uint32_t, uint64_t>> fn_bytes;    // function (index into OpenClass::fns), bytes of it in this batch
  std::vector<StageCopy> unstage;   // ring -> pageable destinations, once the batch is complete
};

// A few helper threads that copy pageable bytes into the ring; the feeder takes part.
class StagePool {
 public:
  explicit StagePool(unsigned helpers) {
    for (unsigned i = 0; i < helpers; ++i) threads_.emplace_back([this] { work(false); });
  }
  unsigned helpers() const { return (unsigned)threads_.size(); }
  ~StagePool() {
    {
      std::lock_guard<std::mutex> lock(mu_);
      quit_ = true;
    }
    cv_.notify_all();
    for (std::thread &t : threads_) t.join();
  }
  void run(const std::vector<StageCopy> &copies) {
    if (copies.empty()) return;
    {
      std::lock_guard<std::mutex> lock(mu_);
      copies_ = &copies;
      next_ = 0;
      left_ = copies.size();
    }
    cv_.notify_all();
    work(true);
    std::unique_lock<std::mutex> lock(mu_);
    done_.wait(lock, [this] { return left_ == 0; });
    copies_ = nullptr;
  }

 private:
  void work(bool caller) {
    std::unique_lock<std::mutex> lock(mu_);
    for (;;) {
      if (copies_ != nullptr && next_ < copies_->size()) {
        const StageCopy c = (*copies_)[next_++];
        lock.unlock();
        stage_copy(c.dst, c.src, c.n);
        lock.lock();
        if (--left_ == 0) done_.notify_all();
        continue;
      }
      if (caller || quit_) return;
      cv_.wait(lock);
    }
  }
  std::mutex mu_;
  std::condition_variable cv_, done_;
  std::vector<std::thread> threads_;
  const std::vector<StageCopy> *copies_ = nullptr;
  size_t next_ = 0, left_ = 0;
  bool quit_ = false;
};

// A parked thread that runs one task at a time: a feeder borrows one for the life of its
// class's sequence instead of creating a thread of its own.
class Worker {
 public:
  Worker() : thread_([this] { loop(); }) {}
  ~Worker() {
    {
      std::lock_guard<std::mutex> lock(mu_);
      quit_ = true;
    }
    cv_.notify_all();
    thread_.join();
  }
  void start(std::function<void()> task) {
    {
      std::lock_guard<std::mutex> lock(mu_);
      task_ = std::move(task);
      busy_ = true;
    }
    cv_.notify_all();
  }
  void wait_idle() {
    std::unique_lock<std::mutex> lock(mu_);
    idle_.wait(lock, [this] { return !busy_; });
  }

 private:
  void loop() {
    std::unique_lock<std::mutex> lock(mu_);
    for (;;) {
      cv_.wait(lock, [this] { return quit_ || task_; });
      if (quit_) return;
      std::function<void()> task = std::move(task_);
      task_ = nullptr;
      lock.unlock();
      task();
      lock.lock();
      busy_ = false;
      idle_.notify_all();
    }
  }
  std::mutex mu_;
  std::condition_variable cv_, idle_;
  std::function<void()> task_;
  bool busy_ = false, quit_ = false;
  std::thread thread_;  // last: the members above exist before the thread looks at them
};

// Threads between jobs. Creating a feeder and three staging helpers costs more than moving a
// small transfer (64 KiB from pageable memory: 143 us with fresh threads per job), so they
// are parked here when a sequence ends and handed to the next one. Never destroyed: parked
// threads simply end with the process.
struct ThreadCache {
  std::mutex mu;
  std::vector<std::unique_ptr<Worker>> workers;
  std::vector<std::unique_ptr<StagePool>> stagers;
};
ThreadCache &thread_cache() {
  static ThreadCache *cache = new ThreadCache();
  return *cache;
}
constexpr size_t kMaxParkedWorkers = 12, kMaxParkedStagers = 6;

std::unique_ptr<Worker> get_worker() {
  ThreadCache &tc = thread_cache();
  {
    std::lock_guard<std::mutex> lock(tc.mu);
    if (!tc.workers.empty()) {
      std::unique_ptr<Worker> w = std::move(tc.workers.back());
      tc.workers.pop_back();
      return w;
    }
  }
  return std::unique_ptr<Worker>(new Worker());
}

void put_worker(std::unique_ptr<Worker> w) {
  if (!w) return;
  ThreadCache &tc = thread_cache();
  std::unique_lock<std::mutex> lock(tc.mu);
  if (tc.workers.size() < kMaxParkedWorkers) {
    tc.workers.push_back(std::move(w));
    return;
  }
  lock.unlock();
  w.reset();  // joins
}

std::unique_ptr<StagePool> get_stagers(unsigned helpers) {
  ThreadCache &tc = thread_cache();
  {
    std::lock_guard<std::mutex> lock(tc.mu);
    for (size_t i = 0; i < tc.stagers.size(); ++i)
      if (tc.stagers[i]->helpers() == helpers) {
        std::unique_ptr<StagePool> sp = std::move(tc.stagers[i]);
        tc.stagers.erase(tc.stagers.begin() + (long)i);
        return sp;
      }
  }
  return std::unique_ptr<StagePool>(new StagePool(helpers));
}

void put_stagers(std::unique_ptr<StagePool> sp) {
  if (!sp) return;
  ThreadCache &tc = thread_cache();
  std::unique_lock<std::mutex> lock(tc.mu);
  if (tc.stagers.size() >= kMaxParkedStagers) {
    // make room by dropping the oldest: thread counts in use change rarely
    std::unique_ptr<StagePool> old = std::move(tc.stagers.front());
    tc.stagers.erase(tc.stagers.begin());
    tc.stagers.push_back(std::move(sp));
    lock.unlock();
    old.reset();  // joins its helpers
    return;
  }
  tc.stagers.push_back(std::move(sp));
}

struct BatchRec {
  uint64_t job;
  uint32_t func;
  uint32_t chunk;
  uint32_t batch;
};

// FT_LOG: one ticket as the copy kernel recorded it, with the job and function (index inside that
// job) that the function-table index of the kernel's decode stands for.
struct OpenLogRec {
  LogEntry e;
  uint64_t job;
  uint32_t func;
  uint32_t batch;
};

struct OpenClass {
  bool used = false;
  bool closed = false;              // ran dry: no batch left to trigger, feeder gone
  std::vector<OpenFn> fns;
  std::shared_ptr<Generation> gen;  // the order in force
  std::deque<OpenBatch> inflight;
  uint64_t batches_triggered = 0;
  uint64_t batches_done = 0;        // of them, seen complete (bytes in place)
  // chunks per batch of this class. The paper's batch (5 chunks of 2 MB) is sized for a PCIe
  // link, where it is a fraction of a millisecond; the on-device class moves a chunk about
  // sixty times faster and a launch per 5 chunks would be all launch cost (8 GiB between
  // slabs, payload rate against 3.3 TB/s for a closed job: 2.7 TB/s at 80 chunks a batch,
  // 3.1 at 320), so its batches hold 64 times as many chunks - 0.2 ms each, a quarter of
  // what five 2 MB chunks take on the paper's PCIe link.
  uint32_t batch_chunks = 5;
  uint64_t tile_bytes = 0;
  uint32_t tiles_per_chunk = 0;
  uint32_t workgroups = 0;
  uint64_t tickets = 0;
  double kernel_ms = 0;
  std::vector<BatchRec> order;
  std::vector<OpenLogRec> log;      // FT_LOG: tickets of the orders already retired, in trigger order
  // staging ring, present once a function with pageable sources has joined
  char *ring = nullptr;
  uint64_t ring_cap = 0, ring_slots = 0;
  uint64_t staged_bytes = 0;
  double stage_ms = 0;
  std::unique_ptr<StagePool> stagers;
  std::unique_ptr<Worker> feeder;   // runs feeder_main for this class until the sequence is dry
};

}  // namespace

struct OpenState {
  std::mutex mu;
  std::condition_variable cv;
  ft_pool *pool = nullptr;
  uint64_t chunk_bytes = 0;
  uint32_t batch_chunks = 5;
  uint32_t depth = 3;               // batches queued ahead of the device
  uint32_t flags = 0;
  OpenClass cls[FT_NCLASS];
  std::unordered_map<uint64_t, uint64_t> left;      // job id -> chunks not yet complete
  std::unordered_map<uint64_t, uint64_t> arrival;   // job id << 2 | class -> batches triggered when it joined
  int error = FT_OK;
  std::string error_text;

  ~OpenState() {
    for (OpenClass &c : cls) {
      if (c.feeder) c.feeder->wait_idle();
      put_worker(std::move(c.feeder));
      put_stagers(std::move(c.stagers));
      put_pinned(pool, c.ring, c.ring_cap);
    }
  }
};

namespace {

void set_error(OpenState *st, hipError_t e, const char *what) {
  if (st->error == FT_OK) {
    st->error = FT_EHIP;
    st->error_text = std::string(what) + ": " + hipGetErrorString(e);
  }
}

// First ticket of chunk rank r in the generation's numbering, and where the empty-tile
// cursor stands there.
void ticket_of_rank(const Generation &g, uint32_t tpc, uint64_t rank, uint64_t *ticket, uint32_t *skip_idx,
                    uint64_t *skip_acc) {
  uint64_t t = rank * tpc, acc = 0;
  uint32_t j = 0;
  // run j starts inside a chunk of rank (at_j + acc_j) / tpc; it lies before `rank` iff that is smaller
  while (j < g.skips.size() && (g.skips[j].at + acc) / tpc < rank) {
    acc += g.skips[j].gap;
    ++j;
  }
  *ticket = t - acc;
  *skip_idx = j;
  *skip_acc = acc;
}

// Tables of the order over everything not yet triggered; uploaded on `user`.
int build_generation(ft_pool *p, OpenState *st, int c, hipStream_t user, std::shared_ptr<Generation> *out) {
  OpenClass &oc = st->cls[c];
  std::shared_ptr<Generation> g(new Generation());
  ClassPlan &cp = g->plan;
  for (uint32_t i = 0; i < oc.fns.size(); ++i) {
    const OpenFn &fn = oc.fns[i];
    if (fn.next_chunk >= fn.nchunks) continue;
    Func f{};
    f.stream_bytes = fn.stream_bytes;
    f.nchunks = fn.nchunks - fn.next_chunk;
    f.func = i;
    f.weight = fn.weight;
    f.desc_off = (uint32_t)cp.xfers.size();
    f.ndesc = (uint32_t)fn.xfers.size();
    f.chunk_base = fn.next_chunk;
    cp.xfers.insert(cp.xfers.end(), fn.xfers.begin(), fn.xfers.end());
    cp.payload += fn.stream_bytes;
    cp.funcs.push_back(f);
  }
  int rc = build_phases(cp.funcs, cp.phases, cp.slots, &cp.nchunks);
  if (rc != FT_OK) return rc;
  build_chunk_table(cp, st->chunk_bytes, oc.tile_bytes, oc.tiles_per_chunk);
  build_skips(cp, st->chunk_bytes, oc.tile_bytes, oc.tiles_per_chunk, &g->skips, &g->ntickets);
  const uint64_t ncounters = (cp.nchunks + oc.batch_chunks - 1) / oc.batch_chunks;
  const Layout lay = layout_of(cp, 0, ncounters);
  rc = get_blob(p, lay.end, true, &g->blob);
  if (rc != FT_OK) return rc;
  std::memset(g->blob.host, 0, lay.end);
  fill_tables(cp, lay, g->blob.host, g->blob.dev, &g->table);
  copy_table(g->blob.host + lay.skips, g->skips);
  g->table.nskips = (uint32_t)g->skips.size();
  g->table.chunk_bytes = st->chunk_bytes;
  g->table.tile_bytes = oc.tile_bytes;
  g->table.tiles_per_chunk = oc.tiles_per_chunk;
  if (st->flags & FT_LOG) {
    rc = get_blob(p, g->ntickets * sizeof(LogEntry) + ncounters * oc.workgroups * sizeof(WgLogEntry), false, &g->log);
    if (rc != FT_OK) {
      put_blob(p, g->blob);
      return rc;
    }
  }
  rc = get_event(p, false, &g->uploaded);
  if (rc != FT_OK) {
    put_blob(p, g->blob);
    put_blob(p, g->log);
    return rc;
  }
  hipError_t e = hipMemcpyAsync(g->blob.dev, g->blob.host, lay.end, hipMemcpyHostToDevice, user);
  if (e == hipSuccess) e = hipEventRecord(g->uploaded, user);
  if (e != hipSuccess) {
    // the copy may have been queued: drain before the buffers are recycled
    (void)hipStreamSynchronize(user);
    put_event(p, false, g->uploaded);
    put_blob(p, g->blob);
    put_blob(p, g->log);
    p->hip_error = std::string("open job table upload: ") + hipGetErrorString(e);
    return FT_EHIP;
  }
  *out = g;
  return FT_OK;
}

void drop_generation(ft_pool *p, Generation *g) {
  put_event(p, false, g->uploaded);
  put_blob(p, g->blob);
  put_blob(p, g->log);
}

// An order is retired (none of its batches is in flight any more): with FT_LOG, what the copy
// kernel recorded for the tickets it triggered is taken over first. Called with st->mu held.
void retire_generation(ft_pool *p, OpenState *st, int c, Generation *g) {
  OpenClass &oc = st->cls[c];
  if (g->log.dev != nullptr && !g->triggered.empty()) {
    const uint64_t t_lo = g->triggered.front().t0, t_hi = g->triggered.back().t1;
    std::vector<LogEntry> host(t_hi - t_lo);
    if (hipMemcpy(host.data(), g->log.dev + t_lo * sizeof(LogEntry), host.size() * sizeof(LogEntry),
                  hipMemcpyDeviceToHost) == hipSuccess) {
      for (const Generation::Triggered &tr : g->triggered)
        for (uint64_t t = tr.t0; t < tr.t1; ++t) {
          OpenLogRec rec;
          rec.e = host[t - t_lo];
          rec.batch = tr.batch;
          const uint32_t fl = rec.e.fl;
          if (fl < g->plan.funcs.size()) {
            const OpenFn &fn = oc.fns[g->plan.funcs[fl].func];
            rec.job = fn.job;
            rec.func = fn.func;
          } else {
            rec.job = 0;
            rec.func = UINT32_MAX;
          }
          oc.log.push_back(rec);
        }
    }
  }
  drop_generation(p, g);
}

constexpr uint64_t kStagePiece = 256 * 1024;  // longest single copy handed to a helper
constexpr uint32_t kOnDeviceBatchScale = 64;  // see OpenClass::batch_chunks

struct Prepared {
  OpenBatch batch;
  ClassTable T;
  uint32_t workgroups = 0;
  bool wait_upload = false;
  std::vector<StageCopy> copies;
};

// Copies between chunk (f, k)'s ring slot and the pageable memory of its staged descriptors:
// `in` brings pageable sources into the slot before the launch, `out` takes what the device
// wrote for pageable destinations away after it.
void stage_chunk(const ClassPlan &cp, const Func &f, uint64_t k, uint64_t chunk_bytes, char *slot,
                 std::vector<StageCopy> *in, std::vector<StageCopy> *out, uint64_t *bytes) {
  const uint64_t c0 = k * chunk_bytes;
  const uint64_t c1 = std::min(c0 + chunk_bytes, f.stream_bytes);
  uint32_t x = find_xfer(cp.xfers.data(), f.desc_off, f.desc_off + f.ndesc - 1, c0);
  for (uint64_t pos = c0; pos < c1; ++x) {
    const Xfer &X = cp.xfers[x];
    const uint64_t q = pos - X.stream_off;
    uint64_t take = X.row_bytes * X.rows - q;
    if (take > c1 - pos) take = c1 - pos;
    if (X.staged) {
      // rows of the descriptor, packed in stream order at offset (stream position - c0) of the slot
      const bool inward = (X.staged & kStagedSrc) != 0;
      const uint64_t base = inward ? X.src : X.dst, pitch = inward ? X.src_pitch : X.dst_pitch;
      uint64_t r = q / X.row_bytes, c = q % X.row_bytes, left = take, at = pos - c0;
      while (left > 0) {
        uint64_t n = std::min(X.row_bytes - c, left);
        char *mem = reinterpret_cast<char *>(base + r * pitch + c);
        *bytes += n;
        left -= n;
        for (uint64_t o = 0; o < n; o += kStagePiece) {
          const uint64_t m = std::min(kStagePiece, n - o);
          if (inward) in->push_back(StageCopy{slot + at + o, mem + o, m});
          else out->push_back(StageCopy{mem + o, slot + at + o, m});
        }
        at += n;
        r += 1;
        c = 0;
      }
    }
    pos += take;
  }
}

// Decides the next batch of class c and books it (ranks, counter, what it holds).
// Called with st->mu held.
bool prepare_batch(OpenState *st, int c, Prepared *out) {
  ft_pool *p = st->pool;
  OpenClass &oc = st->cls[c];
  Generation &g = *oc.gen;
  const ClassPlan &cp = g.plan;
  const uint64_t r0 = g.next_rank;
  const uint64_t r1 = std::min<uint64_t>(r0 + oc.batch_chunks, cp.nchunks);
  ClassTable &T = out->T;
  T = g.table;
  uint64_t t0, t1, acc1;
  uint32_t idx1;
  ticket_of_rank(g, oc.tiles_per_chunk, r0, &t0, &T.skip0, &T.skip_acc0);
  if (r1 == cp.nchunks) t1 = g.ntickets;
  else ticket_of_rank(g, oc.tiles_per_chunk, r1, &t1, &idx1, &acc1);
  T.ticket_base = t0;
  T.ntickets = t1;
  T.ticket = g.table.ticket + g.next_counter;
  {
    uint32_t lo = 0, hi = (uint32_t)cp.phases.size();
    while (hi - lo > 1) {
      const uint32_t mid = (lo + hi) >> 1;
      if (cp.phases[mid].rank_base <= r0) lo = mid; else hi = mid;
    }
    T.phase0 = lo;
  }
  set_cursor_start(T, cp.phases.data(), (uint32_t)cp.phases.size(), g.skips.data(), (uint32_t)g.skips.size());
  const uint64_t slot0 = oc.ring_slots ? (oc.batches_triggered % (st->depth + 1)) * oc.batch_chunks : 0;
  T.stage_base = reinterpret_cast<uint64_t>(oc.ring);
  T.stage_rank0 = r0;
  T.stage_slot0 = slot0;
  if (g.log.dev != nullptr) {
    T.log = reinterpret_cast<LogEntry *>(g.log.dev);
    T.wg_log = reinterpret_cast<WgLogEntry *>(g.log.dev + g.ntickets * sizeof(LogEntry)) +
               (uint64_t)g.next_counter * oc.workgroups;
  }
  OpenBatch &b = out->batch;
  b.gen = oc.gen;
  b.lane = (uint32_t)(oc.batches_triggered & 1);
  const bool timing = (st->flags & FT_TIMING) != 0;
  if (get_event(p, false, &b.done) != FT_OK || (timing && (get_event(p, true, &b.t_begin) != FT_OK ||
                                                           get_event(p, true, &b.t_end) != FT_OK))) {
    if (st->error == FT_OK) st->error = FT_EHIP, st->error_text = p->hip_error;
    put_event(p, false, b.done);
    put_event(p, true, b.t_begin);
    put_event(p, true, b.t_end);
    return false;
  }
  out->wait_upload = !g.waited_upload[b.lane];
  g.waited_upload[b.lane] = true;
  uint64_t wg = oc.workgroups;
  if (wg > t1 - t0) wg = t1 - t0;
  out->workgroups = (uint32_t)wg;
  // what the batch holds, on the host: advances every function's count of triggered chunks
  const uint32_t batch_no = (uint32_t)oc.batches_triggered;
  for (uint64_t r = r0; r < r1; ++r) {
    const ChunkId id = decode_rank(cp.phases.data(), (uint32_t)cp.phases.size(), cp.slots.data(), r);
    const Func &f = cp.funcs[id.fl];
    OpenFn &fn = oc.fns[f.func];
    const uint64_t k = f.chunk_base + id.k;
    fn.next_chunk = k + 1;
    bool found = false;
    for (auto &jc : b.job_chunks)
      if (jc.first == fn.job) jc.second += 1, found = true;
    if (!found) b.job_chunks.push_back({fn.job, 1});
    {
      const uint64_t c0 = k * st->chunk_bytes;
      const uint64_t n = std::min(st->chunk_bytes, fn.stream_bytes - c0);
      if (!b.fn_bytes.empty() && b.fn_bytes.back().first == f.func) b.fn_bytes.back().second += n;
      else b.fn_bytes.push_back({f.func, n});
    }
    if (st->flags & FT_KEEP) oc.order.push_back(BatchRec{fn.job, fn.func, (uint32_t)k, batch_no});
    if (fn.staged)
      stage_chunk(cp, f, k, st->chunk_bytes, oc.ring + (slot0 + (r - r0)) * st->chunk_bytes, &out->copies,
                  &b.unstage, &oc.staged_bytes);
  }
  if (g.log.dev != nullptr) g.triggered.push_back(Generation::Triggered{t0, t1, batch_no});
  g.next_rank = r1;
  g.next_counter += 1;
  g.inflight += 1;
  oc.tickets += t1 - t0;
  oc.batches_triggered += 1;
  return true;
}

// Launches a prepared batch; only the class's feeder thread launches, so batches reach
// their streams in order. Called without st->mu.
hipError_t launch_batch(ft_pool *p, int c, Prepared &pr) {
  OpenBatch &b = pr.batch;
  hipStream_t s = b.lane ? p->ctx->alt_streams[c] : p->ctx->streams[c];
  if (c == FT_P2P && b.lane) {
    // the class's second stream may share its hardware queue with a host-link stream: while a host-link
    // kernel of a detached closed job runs, the batch queues behind its predecessor instead
    std::lock_guard<std::mutex> ctx_lock(p->ctx->mu);
    if (p->ctx->hostlink_marker != nullptr && hipEventQuery(p->ctx->hostlink_marker) == hipErrorNotReady) s = p->ctx->streams[c];
  }
  hipError_t e = hipSuccess;
  if (pr.wait_upload) e = hipStreamWaitEvent(s, b.gen->uploaded, 0);
  if (e == hipSuccess) e = launch_copy(pr.T, c, pr.workgroups, s, b.t_begin, b.t_end);
  if (e == hipSuccess) e = hipEventRecord(b.done, s);
  return e;
}

void feeder_main(OpenState *st, int c) {
  ft_pool *p = st->pool;
  (void)hipSetDevice(p->device);
  OpenClass &oc = st->cls[c];
  std::unique_lock<std::mutex> lock(st->mu);
  // the chunks of a batch are complete: the jobs they belong to are told (lock held)
  auto count_done = [&](const OpenBatch &b) {
    for (auto &fb : b.fn_bytes) oc.fns[fb.first].done_bytes += fb.second;
    oc.batches_done += 1;
    for (auto &jc : b.job_chunks) {
      auto it = st->left.find(jc.first);
      if (it != st->left.end()) it->second = it->second > jc.second ? it->second - jc.second : 0;
    }
    st->cv.notify_all();
  };
  OpenBatch carry;  // complete on the device, its bytes still to be taken out of the ring
  bool have_carry = false;
  for (;;) {
    while (st->error == FT_OK && oc.inflight.size() < st->depth && oc.gen->next_rank < oc.gen->plan.nchunks) {
      Prepared pr;
      if (!prepare_batch(st, c, &pr)) break;
      StagePool *stagers = oc.stagers.get();
      lock.unlock();
      // the ring slots of this batch were last used depth + 1 batches ago; at most depth - 1
      // batches are in flight, so that one is complete
      if (!pr.copies.empty()) {
        const auto s0 = std::chrono::steady_clock::now();
        stagers->run(pr.copies);
        const double ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - s0).count();
        lock.lock();
        oc.stage_ms += ms;
        lock.unlock();
      }
      const hipError_t e = launch_batch(p, c, pr);
      lock.lock();
      if (e != hipSuccess) {
        set_error(st, e, "open job batch launch");
        put_event(p, false, pr.batch.done);
        put_event(p, true, pr.batch.t_begin);
        put_event(p, true, pr.batch.t_end);
        pr.batch.gen->inflight -= 1;
        break;
      }
      oc.inflight.push_back(std::move(pr.batch));
    }
    if (have_carry) {
      // A complete batch whose ring slots hold bytes for pageable destinations. The batch
      // that follows the ones in flight has just been launched (above), so the link stays
      // busy while these bytes go on to where they belong. Their slots are handed out again
      // only to a batch that this thread prepares later.
      StagePool *stagers = oc.stagers.get();
      lock.unlock();
      const auto s0 = std::chrono::steady_clock::now();
      stagers->run(carry.unstage);
      const double ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - s0).count();
      lock.lock();
      oc.stage_ms += ms;
      count_done(carry);
      have_carry = false;
      continue;
    }
    if (oc.inflight.empty()) {
      // dry (or failed): later arrivals start a sequence of their own
      oc.closed = true;
      retire_generation(p, st, c, oc.gen.get());
      // chunks that will never be triggered count as done so that no waiter hangs
      if (st->error != FT_OK) {
        for (auto &kv : st->left) kv.second = 0;
      }
      st->cv.notify_all();
      return;
    }
    OpenBatch b = std::move(oc.inflight.front());
    oc.inflight.pop_front();
    lock.unlock();
    hipError_t e = hipEventSynchronize(b.done);
    float ms = 0;
    if (e == hipSuccess && b.t_begin != nullptr) e = hipEventElapsedTime(&ms, b.t_begin, b.t_end);
    lock.lock();
    if (e != hipSuccess) set_error(st, e, "open job batch");
    oc.kernel_ms += ms;
    put_event(p, false, b.done);
    put_event(p, true, b.t_begin);
    put_event(p, true, b.t_end);
    b.gen->inflight -= 1;
    if (b.gen->inflight == 0 && b.gen != oc.gen) retire_generation(p, st, c, b.gen.get());
    if (st->error == FT_OK && !b.unstage.empty()) {
      carry = std::move(b);
      have_carry = true;
    } else {
      count_done(b);
    }
  }
}

// Pinned ring and helper threads for class c, once, when the first function with pageable
// memory on its host side joins.
int ensure_ring(ft_pool *p, OpenState *st, int c) {
  OpenClass &oc = st->cls[c];
  if (oc.ring != nullptr) return FT_OK;
  const uint64_t slots = (uint64_t)(st->depth + 1) * oc.batch_chunks;
  int rc = get_pinned(p, slots * st->chunk_bytes, &oc.ring, &oc.ring_cap);
  if (rc != FT_OK) return rc;
  oc.ring_slots = slots;
  oc.stagers = get_stagers(p->stage_threads ? p->stage_threads - 1 : 3);
  return FT_OK;
}

bool any_staged(const ClassPlan &cp) {
  for (const Xfer &x : cp.xfers)
    if (x.staged != 0) return true;
  return false;
}

void add_functions(OpenClass &oc, uint64_t job_id, const ClassPlan &cp) {
  for (const Func &f : cp.funcs) {
    OpenFn fn;
    fn.job = job_id;
    fn.func = f.func;
    fn.weight = f.weight;  // the caller's weight (the callers below undo the gcd reduction of planning)
    fn.stream_bytes = f.stream_bytes;
    fn.nchunks = f.nchunks;
    fn.next_chunk = 0;
    fn.xfers.assign(cp.xfers.begin() + f.desc_off, cp.xfers.begin() + f.desc_off + f.ndesc);
    fn.staged = false;
    for (const Xfer &x : fn.xfers) fn.staged = fn.staged || x.staged != 0;
    oc.fns.push_back(std::move(fn));
  }
}

}  // namespace

void run_host_copies(ft_pool *p, const std::vector<HostCopy> &copies) {
  uint64_t total = 0;
  for (const HostCopy &c : copies) total += c.n;
  if (total < 2 * kStagePiece) {
    for (const HostCopy &c : copies) stage_copy(c.dst, c.src, c.n);
    return;
  }
  std::vector<StageCopy> pieces;
  for (const HostCopy &c : copies)
    for (uint64_t o = 0; o < c.n; o += kStagePiece)
      pieces.push_back(StageCopy{c.dst + o, c.src + o, std::min(kStagePiece, c.n - o)});
  std::unique_ptr<StagePool> stagers = get_stagers(p->stage_threads ? p->stage_threads - 1 : 3);
  stagers->run(pieces);
  put_stagers(std::move(stagers));
}

int open_submit(ft_pool *p, Job *job, SubmitPlan &plan, const uint32_t *weights, uint64_t chunk_bytes,
                hipStream_t user) {
  std::shared_ptr<OpenState> st(new OpenState());
  st->pool = p;
  st->chunk_bytes = chunk_bytes;
  st->batch_chunks = p->batch_chunks ? p->batch_chunks : 5;
  st->depth = p->batch_depth ? p->batch_depth : 3;
  st->flags = job->flags;
  uint64_t chunks = 0;
  const bool with_p2p = plan.cls[FT_P2P].nchunks > 0;
  std::unique_lock<std::mutex> lock(st->mu);
  // no feeder runs yet: a failure only has to hand back the tables built so far
  auto undo = [&](int rc) {
    bool drained = false;
    for (OpenClass &oc : st->cls)
      if (oc.gen) {
        if (!drained) (void)hipStreamSynchronize(user);  // its upload may still be queued
        drained = true;
        drop_generation(p, oc.gen.get());
      }
    return rc;
  };
  for (int c = 0; c < FT_NCLASS; ++c) {
    ClassPlan &cp = plan.cls[c];
    if (cp.nchunks == 0) continue;
    OpenClass &oc = st->cls[c];
    oc.used = true;
    oc.batch_chunks = st->batch_chunks * (c == FT_P2P ? kOnDeviceBatchScale : 1u);
    // the caller's weights, not the gcd-reduced ones: functions of later jobs are weighed against them
    for (Func &f : cp.funcs) f.weight = weights[f.func];
    add_functions(oc, job->id, cp);
    if (any_staged(cp)) {
      int rc = ensure_ring(p, st.get(), c);
      if (rc != FT_OK) return undo(rc);
    }
    const Tuning &tn = p->tuning[c];
    tile_shape(chunk_bytes, tn.tile_bytes ? tn.tile_bytes : default_tile(c, with_p2p, mostly_short_rows(cp), ~0ull),
               &oc.tile_bytes, &oc.tiles_per_chunk);
    oc.workgroups = tn.workgroups ? tn.workgroups : default_workgroups(p, c, with_p2p);
    // consecutive batches overlap on the class's two streams, so each launch gets a share of
    // the host link's in-flight budget: 16 workgroups (contended workload, batches of 2.5 MiB:
    // 50 GB/s with 64 workgroups per launch, 57 with 16)
    if (!tn.workgroups && c != FT_P2P) oc.workgroups = 16;
    int rc = build_generation(p, st.get(), c, user, &oc.gen);
    if (rc != FT_OK) return undo(rc);
    chunks += cp.nchunks;
    st->arrival[job->id << 2 | (uint64_t)c] = 0;
  }
  st->left[job->id] = chunks;
  for (int c = 0; c < FT_NCLASS; ++c)
    if (st->cls[c].used) {
      OpenState *raw = st.get();  // outlives the task: ~OpenState waits for the feeders
      st->cls[c].feeder = get_worker();
      st->cls[c].feeder->start([raw, c] { feeder_main(raw, c); });
    }
  lock.unlock();
  job->open = st;
  return FT_OK;
}

int open_merge(ft_pool *p, Job *open_job, Job *job, SubmitPlan &plan, const uint32_t *weights,
               hipStream_t user) {
  std::shared_ptr<OpenState> st = open_job->open;
  if (!st) return FT_EINVAL;
  std::unique_lock<std::mutex> lock(st->mu);
  if (st->error != FT_OK) {
    p->hip_error = st->error_text;
    return st->error;
  }
  // all or nothing: every class the newcomer uses must still have batches to trigger
  for (int c = 0; c < FT_NCLASS; ++c)
    if (plan.cls[c].nchunks > 0 && (!st->cls[c].used || st->cls[c].closed)) return FT_ECLOSED;
  // Build the new order of every class first and put it in force only when all of them
  // exist, so that a failure half way leaves the sequence as it was (the feeders cannot
  // look while the lock is held).
  struct Pending {
    int c;
    size_t fns_before;
    std::shared_ptr<Generation> gen;
  };
  std::vector<Pending> pending;
  auto roll_back = [&](int rc) {
    bool drained = false;
    for (Pending &pd : pending) {
      st->cls[pd.c].fns.resize(pd.fns_before);
      if (pd.gen) {
        if (!drained) (void)hipStreamSynchronize(user);  // its upload may still be queued
        drained = true;
        drop_generation(p, pd.gen.get());
      }
    }
    return rc;
  };
  uint64_t chunks = 0;
  for (int c = 0; c < FT_NCLASS; ++c) {
    ClassPlan &cp = plan.cls[c];
    if (cp.nchunks == 0) continue;
    OpenClass &oc = st->cls[c];
    for (Func &f : cp.funcs) f.weight = weights[f.func];
    pending.push_back(Pending{c, oc.fns.size(), nullptr});
    add_functions(oc, job->id, cp);
    int rc = any_staged(cp) ? ensure_ring(p, st.get(), c) : FT_OK;
    if (rc == FT_OK) rc = build_generation(p, st.get(), c, user, &pending.back().gen);
    if (rc != FT_OK) return roll_back(rc);
    chunks += cp.nchunks;
  }
  for (Pending &pd : pending) {
    OpenClass &oc = st->cls[pd.c];
    std::shared_ptr<Generation> old = oc.gen;
    oc.gen = pd.gen;
    if (old->inflight == 0) retire_generation(p, st.get(), pd.c, old.get());
    st->arrival[job->id << 2 | (uint64_t)pd.c] = oc.batches_triggered;
  }
  st->left[job->id] = chunks;
  lock.unlock();
  st->cv.notify_all();
  job->open = st;
  return FT_OK;
}

int open_reweight(ft_pool *p, Job *job, const uint32_t *weights, hipStream_t user, uint64_t *batch_out) {
  std::shared_ptr<OpenState> st = job->open;
  if (!st) return FT_EINVAL;
  std::unique_lock<std::mutex> lock(st->mu);
  if (st->error != FT_OK) {
    p->hip_error = st->error_text;
    return st->error;
  }
  // As for a merge: the new order of every class is built first and put in force only when
  // all of them exist; a failure half way restores the old weights.
  struct Pending {
    int c;
    std::vector<std::pair<uint32_t, uint32_t>> old_weights;  // index into fns, weight before
    std::shared_ptr<Generation> gen;
  };
  std::vector<Pending> pending;
  auto roll_back = [&](int rc) {
    bool drained = false;
    for (Pending &pd : pending) {
      for (auto &ow : pd.old_weights) st->cls[pd.c].fns[ow.first].weight = ow.second;
      if (pd.gen) {
        if (!drained) (void)hipStreamSynchronize(user);  // its upload may still be queued
        drained = true;
        drop_generation(p, pd.gen.get());
      }
    }
    return rc;
  };
  for (int c = 0; c < FT_NCLASS; ++c) {
    batch_out[c] = UINT64_MAX;
    OpenClass &oc = st->cls[c];
    if (!oc.used || oc.closed || oc.gen->next_rank >= oc.gen->plan.nchunks) continue;  // nothing left to reorder
    Pending pd{c, {}, nullptr};
    bool differs = false;
    for (uint32_t i = 0; i < oc.fns.size(); ++i) {
      OpenFn &fn = oc.fns[i];
      if (fn.job != job->id || fn.next_chunk >= fn.nchunks) continue;
      pd.old_weights.push_back({i, fn.weight});
      differs = true;
    }
    if (!differs) continue;  // every chunk of the job in this class has been triggered
    pending.push_back(std::move(pd));
    for (auto &ow : pending.back().old_weights) oc.fns[ow.first].weight = weights[oc.fns[ow.first].func];
    int rc = build_generation(p, st.get(), c, user, &pending.back().gen);
    if (rc != FT_OK) return roll_back(rc);
  }
  for (Pending &pd : pending) {
    OpenClass &oc = st->cls[pd.c];
    std::shared_ptr<Generation> old = oc.gen;
    oc.gen = pd.gen;
    if (old->inflight == 0) retire_generation(p, st.get(), pd.c, old.get());
    batch_out[pd.c] = oc.batches_triggered;
  }
  return FT_OK;
}

int open_wait(ft_pool *p, const std::shared_ptr<OpenState> &st, uint64_t job_id) {
  std::unique_lock<std::mutex> lock(st->mu);
  st->cv.wait(lock, [&] {
    auto it = st->left.find(job_id);
    return it == st->left.end() || it->second == 0;
  });
  if (st->error != FT_OK) {
    p->hip_error = st->error_text;
    return st->error;
  }
  return FT_OK;
}

bool open_done(const std::shared_ptr<OpenState> &st, uint64_t job_id) {
  std::lock_guard<std::mutex> lock(st->mu);
  auto it = st->left.find(job_id);
  return it == st->left.end() || it->second == 0;
}

void open_stats(const std::shared_ptr<OpenState> &st, int c, uint64_t *tickets, uint64_t *tile_bytes,
                uint32_t *workgroups, float *kernel_ms, uint64_t *batches) {
  std::lock_guard<std::mutex> lock(st->mu);
  const OpenClass &oc = st->cls[c];
  *tickets = oc.tickets;
  *tile_bytes = oc.tile_bytes;
  *workgroups = oc.workgroups;
  *kernel_ms = (st->flags & FT_TIMING) ? (float)oc.kernel_ms : -1.f;
  *batches = oc.batches_triggered;
}

int open_arrival(const std::shared_ptr<OpenState> &st, uint64_t job_id, int c, uint64_t *batch) {
  std::lock_guard<std::mutex> lock(st->mu);
  auto it = st->arrival.find(job_id << 2 | (uint64_t)c);
  if (it == st->arrival.end()) return FT_EINVAL;
  *batch = it->second;
  return FT_OK;
}

int open_progress(const std::shared_ptr<OpenState> &st, uint64_t job_id, int c, uint64_t *bytes_done, uint32_t nfunc,
                  uint64_t *batches_done) {
  std::lock_guard<std::mutex> lock(st->mu);
  const OpenClass &oc = st->cls[c];
  for (uint32_t f = 0; f < nfunc; ++f) bytes_done[f] = 0;
  for (const OpenFn &fn : oc.fns)
    if (fn.job == job_id && fn.func < nfunc) bytes_done[fn.func] = fn.done_bytes;
  if (batches_done) *batches_done = oc.batches_done;
  return FT_OK;
}

int open_log(const std::shared_ptr<OpenState> &st, int c, double ns_per_tick, uint64_t *t_begin_ns, uint64_t *t_end_ns,
             uint64_t *job_out, uint32_t *func_out, uint32_t *chunk_out, uint64_t *byte_off_out, uint32_t *bytes_out,
             uint32_t *batch_out, uint64_t cap, uint64_t *n_out) {
  std::lock_guard<std::mutex> lock(st->mu);
  const OpenClass &oc = st->cls[c];
  if (oc.used && !oc.closed) return FT_EBUSY;  // orders still in force hold their part of the log on the device
  *n_out = oc.log.size();
  for (uint64_t t = 0; t < oc.log.size() && t < cap; ++t) {
    const OpenLogRec &r = oc.log[t];
    if (t_begin_ns) t_begin_ns[t] = (uint64_t)(r.e.t_begin * ns_per_tick);
    if (t_end_ns) t_end_ns[t] = (uint64_t)(r.e.t_end * ns_per_tick);
    if (job_out) job_out[t] = r.job;
    if (func_out) func_out[t] = r.func;
    if (chunk_out) chunk_out[t] = (uint32_t)r.e.k;
    if (byte_off_out) byte_off_out[t] = r.e.b0;
    if (bytes_out) bytes_out[t] = (uint32_t)(r.e.b1 - r.e.b0);
    if (batch_out) batch_out[t] = r.batch;
  }
  return FT_OK;
}

uint64_t open_order(const std::shared_ptr<OpenState> &st, int c, uint64_t *job_out, uint32_t *func_out,
                    uint32_t *chunk_out, uint32_t *batch_out, uint64_t cap) {
  std::lock_guard<std::mutex> lock(st->mu);
  const OpenClass &oc = st->cls[c];
  for (uint64_t i = 0; i < oc.order.size() && i < cap; ++i) {
    job_out[i] = oc.order[i].job;
    func_out[i] = oc.order[i].func;
    chunk_out[i] = oc.order[i].chunk;
    batch_out[i] = oc.order[i].batch;
  }
  return oc.order.size();
}

}  // namespace ft
