// Internals shared by the translation units of the library (not part of the C ABI).
#pragma once
#include <hip/hip_runtime_api.h>

#include <cstring>
#include <memory>
#include <mutex>
#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/faastube.h"
#include "ft_kernels.h"
#include "ft_plan.h"
#include "ft_pool.h"
#include "ft_tables.h"

namespace ft {

struct OpenState;  // ft_open.cpp: a job that triggers its chunks in batches and accepts merges

// A device buffer with a pinned host twin of the same size; recycled between jobs so
// that a steady stream of submits allocates nothing.
struct Blob {
  char *dev = nullptr;
  char *host = nullptr;  // null for device-only blobs
  uint64_t cap = 0;
};

struct ClassRun {
  bool used = false;
  ClassTable table{};       // device addresses
  ClassPlan plan;           // host copy (DMA path, log decoding, stats)
  uint64_t tile_bytes = 0;
  uint32_t tiles_per_chunk = 0;
  uint32_t workgroups = 0;
  // pool->pool job of short pitched rows: the kernel's light build, two workgroups per compute unit
  bool light = false;
  bool on_user_stream = false;  // launched on the caller's stream, tables in the launch
  hipStream_t stream = nullptr; // the library's stream it runs on otherwise
  int counter_pair = -1;        // its self-resetting counter pair, if it needed a counter
  // ev_done orders the caller's stream and ft_wait after the class's work. With FT_TIMING,
  // ev_begin / ev_end bracket it: bound to the kernel's dispatch on the kernel path,
  // recorded around the copy calls on the DMA path.
  hipEvent_t ev_begin = nullptr, ev_end = nullptr, ev_done = nullptr;
  Blob log;
  std::vector<Skip> skips;
  std::vector<LogEntry> log_host;
  std::vector<WgLogEntry> wg_log_host;
  float device_ms = -1.f;
  float begin_ms = -1.f, end_ms = -1.f;  // since the device's timing epoch, if one was set before the job
};

// One host copy owed after a job's device work: from the job's bounce buffer to pageable memory.
struct HostCopy {
  char *dst;
  const char *src;
  uint64_t n;
};

struct Job {
  uint64_t id = 0;
  uint32_t flags = 0;
  bool keep = false;
  bool waited = false;
  bool waiting = false;  // a thread is blocked in ft_wait for this job (the pool's mutex is not held then)
  ClassRun run[FT_NCLASS];
  Blob tables;
  std::unique_ptr<InlineBlob> inline_tables;  // a small job's tables, passed with the launch instead
  std::vector<uint64_t> allocs;         // offsets of the pool allocations the job refers to,
  std::vector<uint64_t> alloc_serials;  // and which allocation at that offset it was
  uint64_t chunk_bytes = 0;
  uint32_t nfunc = 0;    // functions the job was submitted with
  double host_submit_us = 0;
  std::shared_ptr<OpenState> open;  // set for a job submitted with FT_OPEN or merged into one
  // a closed job with pageable host sides: pinned buffer that stands in for them, and what
  // ft_wait still has to copy out of it once the device is done
  char *bounce = nullptr;
  uint64_t bounce_cap = 0;
  std::vector<HostCopy> unstage;
  uint64_t class_payload[FT_NCLASS] = {0, 0, 0};
  uint64_t class_chunks[FT_NCLASS] = {0, 0, 0};
};

struct Tuning {
  uint32_t workgroups = 0;
  uint64_t tile_bytes = 0;
};

// Per-device resources shared by every pool on that device and kept for the life of
// the process: one stream per link class (so the three classes sit on three hardware
// queues and really run side by side), recycled table buffers and events. Creating a
// pool therefore costs no HIP call, and a steady stream of submits allocates nothing.
struct DeviceCtx {
  std::mutex mu;
  int device = 0;
  bool ready = false;
  int cu_count = 0;
  int clock_khz = 0;
  hipStream_t streams[FT_NCLASS] = {nullptr, nullptr, nullptr};
  // second stream per class: an open job launches its batches on the two in turn, so the
  // head of one batch overlaps the tail of the one before and the link does not idle
  // (contended workload, batches of 2.5 MiB, 3 queued ahead: 46 -> 50 GB/s)
  hipStream_t alt_streams[FT_NCLASS] = {nullptr, nullptr, nullptr};
  // Detached closed jobs also use both pool->pool streams: their launches are independent of each
  // other (nothing orders two detached jobs), and on one stream every launch would wait for the last
  // workgroup of the one before. A launch goes to the other stream only while the last one is still
  // running (lane_marker, recorded behind every such launch, says so): the process has few hardware
  // queues, streams share them, and a pool->pool launch on a stream that shares its queue with the
  // host->pool stream runs after that stream's kernel instead of beside it (large mixed workload,
  // launches 150 us apart that never meet: taking the streams strictly in turn cost 0.6 % of the
  // aggregate rate for nothing).
  uint32_t detached_lane[FT_NCLASS] = {0, 0, 0};  // stream the last such launch went to; guarded by mu
  hipEvent_t lane_marker[FT_NCLASS] = {nullptr, nullptr, nullptr};
  // recorded behind every host-link kernel of a closed job: while one of them runs, a pool->pool
  // launch stays on the first stream (the second may share its hardware queue with a host-link
  // stream, and would then wait milliseconds for that kernel instead of overlapping a tail)
  hipEvent_t hostlink_marker = nullptr;
  hipEvent_t epoch = nullptr;  // ft_timing_epoch: the instant that ft_job_stats' begin / end times count from
  std::vector<Blob> free_blobs;      // with a pinned twin
  std::vector<Blob> free_dev_blobs;  // device only
  std::vector<hipEvent_t> free_events, free_timing_events;
  std::vector<std::pair<char *, uint64_t>> free_pinned;  // staging rings between jobs
  // a counter nobody reads, for launches in which every ticket has a workgroup of its own
  unsigned long long *idle_counter = nullptr;
  // pairs of self-resetting counters (see ClassTable::self_reset) for jobs whose tables
  // travel with the launch: zero whenever no kernel is using them
  unsigned long long *counter_pairs = nullptr;
  std::vector<uint32_t> free_pairs;
};

DeviceCtx *device_ctx(int device);

}  // namespace ft

struct ft_pool {
  std::mutex mu;
  ft::SlabPool slabs;
  int device;
  std::vector<ft::HostWindow> windows;
  ft::DeviceCtx *ctx;
  std::unordered_map<uint64_t, std::unique_ptr<ft::Job>> jobs;
  uint64_t next_job = 1;
  ft::Tuning tuning[FT_NCLASS];
  uint32_t batch_chunks = 5;  // chunks per triggered batch of an open job (Sec. 6.1 default)
  uint32_t batch_depth = 3;   // batches an open job keeps queued ahead of the device
  uint32_t stage_threads = 4; // threads (the feeder included) that fill the staging ring
  std::string hip_error;

  ft_pool(uint64_t slab_bytes, int dev) : slabs(slab_bytes), device(dev), ctx(ft::device_ctx(dev)) {}
};

namespace ft {

#define FT_HIP(p, call)                                                        \
  do {                                                                         \
    hipError_t e_ = (call);                                                    \
    if (e_ != hipSuccess) {                                                    \
      (p)->hip_error = std::string(#call) + ": " + hipGetErrorString(e_);      \
      return FT_EHIP;                                                          \
    }                                                                          \
  } while (0)

struct DeviceGuard {
  int prev = -1;
  bool ok = false;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) == hipSuccess && prev != dev) ok = hipSetDevice(dev) == hipSuccess;
  }
  ~DeviceGuard() {
    if (ok) (void)hipSetDevice(prev);
  }
};


int ensure_device(ft_pool *p);
// For the store (ft_store.cpp), which carries out its moves as jobs on one stream that it does not
// wait for: jobs not yet waited for that refer to the allocation at `off` (0 if there is none), and
// a free that does not mind them - what reuses the slabs is ordered after those jobs on that stream.
uint32_t slab_busy(ft_pool *p, uint64_t off);
int slab_free_ordered(ft_pool *p, uint64_t off);
int get_blob(ft_pool *p, uint64_t need, bool pinned_twin, Blob *out);
void put_blob(ft_pool *p, Blob &b);
int get_event(ft_pool *p, bool timing, hipEvent_t *out);
void put_event(ft_pool *p, bool timing, hipEvent_t &e);
uint64_t align_up(uint64_t v, uint64_t a);
// Pinned host memory for a staging ring (kept for the life of the process and reused).
int get_pinned(ft_pool *p, uint64_t need, char **out, uint64_t *cap);
void put_pinned(ft_pool *p, char *ptr, uint64_t cap);

// Byte layout of one class's tables inside a table blob.
// A table copied to its place in a blob (memcpy must not be handed the null data() of an empty vector).
template <class T>
inline void copy_table(char *dst, const std::vector<T> &v) {
  if (!v.empty()) std::memcpy(dst, v.data(), v.size() * sizeof(T));
}

struct Layout {
  uint64_t ticket, phases, slots, funcs, xfers, chunks, skips, end;
};
// nbatches: ticket counters to reserve (one per launch that will use these tables)
Layout layout_of(const ClassPlan &cp, uint64_t base, uint64_t ncounters = 1);
// Copies the plan's tables into the host twin at `h` and fills the device pointers of T
// (d = null: offsets from the start of `h`, for tables that travel with the launch).
void fill_tables(const ClassPlan &cp, const Layout &lay, char *h, char *d, ClassTable *T);
// Layout without a ticket counter, from offset 0: for tables that travel with the launch.
Layout inline_layout_of(const ClassPlan &cp);
// fill_tables plus everything of the table header that depends on the tile shape: ticket count,
// runs of empty tiles (copied to `h` as well), cursor start, chunk and tile sizes.
void fill_class_table(const ClassPlan &cp, const Layout &lay, char *h, char *d, const std::vector<Skip> &skips,
                      uint64_t ntickets, uint64_t chunk_bytes, uint64_t tile_bytes, uint32_t tiles_per_chunk,
                      ClassTable *T);

uint32_t default_workgroups(const ft_pool *p, int cls, bool with_p2p);
// payload: bytes of the class in the job (all ones for an open job, whose traffic is not known in advance)
uint64_t default_tile(int cls, bool with_p2p, bool short_rows, uint64_t payload);
bool mostly_short_rows(const ClassPlan &cp);

// ft_open.cpp. All but open_wait are called with the pool's mutex held and the pool's
// device current; open_wait blocks and must be called without the pool's mutex.
int open_submit(ft_pool *p, Job *job, SubmitPlan &plan, const uint32_t *weights, uint64_t chunk_bytes,
                hipStream_t user);
int open_merge(ft_pool *p, Job *open_job, Job *job, SubmitPlan &plan, const uint32_t *weights,
               hipStream_t user);
// Host copies between pageable memory and a pinned buffer; large ones are shared out among the
// parked staging threads (the caller takes part). Takes none of the pool's or the jobs' locks itself.
void run_host_copies(ft_pool *p, const std::vector<HostCopy> &copies);
// New weights (one per function of the job) from the first batch of every class not yet
// triggered; batch_out[FT_NCLASS] receives that batch's number, UINT64_MAX for a class in
// which nothing of the job is left to trigger.
int open_reweight(ft_pool *p, Job *job, const uint32_t *weights, hipStream_t user, uint64_t *batch_out);
int open_wait(ft_pool *p, const std::shared_ptr<OpenState> &st, uint64_t job_id);
bool open_done(const std::shared_ptr<OpenState> &st, uint64_t job_id);  // what open_wait would wait for has happened
void open_stats(const std::shared_ptr<OpenState> &st, int c, uint64_t *tickets, uint64_t *tile_bytes,
                uint32_t *workgroups, float *kernel_ms, uint64_t *batches);
int open_arrival(const std::shared_ptr<OpenState> &st, uint64_t job_id, int c, uint64_t *batch);
// Bytes of each of the job's functions (class c) whose batches have been seen complete so far.
int open_progress(const std::shared_ptr<OpenState> &st, uint64_t job_id, int c, uint64_t *bytes_done, uint32_t nfunc,
                  uint64_t *batches_done);
// FT_LOG of an open sequence: every ticket triggered on class c, in trigger order, as the copy kernel
// recorded it. FT_EBUSY while the class still has batches to trigger or in flight.
int open_log(const std::shared_ptr<OpenState> &st, int c, double ns_per_tick, uint64_t *t_begin_ns, uint64_t *t_end_ns,
             uint64_t *job_out, uint32_t *func_out, uint32_t *chunk_out, uint64_t *byte_off_out, uint32_t *bytes_out,
             uint32_t *batch_out, uint64_t cap, uint64_t *n_out);
uint64_t open_order(const std::shared_ptr<OpenState> &st, int c, uint64_t *job_out, uint32_t *func_out,
                    uint32_t *chunk_out, uint32_t *batch_out, uint64_t cap);

}  // namespace ft
