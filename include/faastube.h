/*
 * faastube.h - C ABI of the single-GPU batched scatter-gather transfer engine.
 *
 * The engine is the data-passing hot path of FaaSTube (arxiv 2411.01830) for
 * one GPU: intermediate tensors of many concurrent functions move between
 * pinned host memory and a pooled GPU store (Sec. 5.1 "Host-GPU"), and between
 * two places of that store (Sec. 5.1 "Intra-GPU"), cut into fixed-size chunks
 * that are interleaved across functions in proportion to per-function weights
 * (Sec. 6.1), with the store handing out memory from a growable pool instead
 * of the native allocator (Sec. 7.1).
 *
 * Conventions for every call
 *   - Returns FT_OK (0) or a negative FT_E* code. On error nothing is launched
 *     and no state changes. ft_strerror() names a code.
 *   - "host pointer" / "device pointer" is stated per argument. The library
 *     never takes ownership of caller memory.
 *   - One mutex per pool: calls on one pool from several threads serialise, except
 *     that ft_wait gives the mutex up while it blocks. ft_pool_destroy must not run
 *     beside any other call on the same pool.
 *   - All multi-byte fields are little endian.
 */
#ifndef FAASTUBE_H
#define FAASTUBE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ft_pool ft_pool; /* opaque; created by ft_pool_create, freed by ft_pool_destroy */
typedef uint64_t ft_off_t;      /* byte offset in a pool's logical offset space */
typedef uint64_t ft_job_t;      /* handle of one submit */

/* address spaces of a descriptor side */
enum {
  FT_HOST = 0,     /* pinned host memory the device can address */
  FT_POOL = 1,     /* the pool's logical offset space */
  FT_PAGEABLE = 2  /* ordinary host memory, as the source of a host->pool or the destination of a
                      pool->host transfer. In open jobs it travels through the circular pinned
                      buffer (Sec. 6.1); a job that is not open may name up to 8 MiB of it, which
                      go through a pinned buffer of the job's own (see ft_pageable_window_add) */
};

/* link classes: each has its own chunk schedule and its own kernel */
enum { FT_H2P = 0, FT_P2H = 1, FT_P2P = 2, FT_NCLASS = 3 };

/* return codes */
enum {
  FT_OK = 0,
  FT_EINVAL = -1,   /* malformed argument (see each call) */
  FT_ENOMEM = -2,   /* no run of free slabs; the caller may ft_pool_grow and retry */
  FT_ERANGE = -3,   /* a pool range is not inside one live allocation, or a host range is
                       outside every registered host window */
  FT_EOVERLAP = -4, /* with FT_VALIDATE: a destination byte is written twice or also read */
  FT_EBUSY = -5,    /* ft_slab_free of an allocation a not-yet-waited job refers to */
  FT_EHIP = -6,     /* a HIP runtime call failed; ft_last_hip_error() gives its text */
  FT_ECLOSED = -7,  /* ft_submit_merge: the open job has no batch left to trigger on a link
                       class the new transfers use; submit them as a job of their own */
  FT_E2BIG = -8     /* ft_submit_static: the schedule tables of one link class exceed the library's
                       fixed device buffer; use ft_submit_transfers */
};

/* flags of ft_submit_transfers */
enum {
  FT_VALIDATE = 1 << 0, /* exact overlap check, O(rows log rows) on the host */
  FT_LOG = 1 << 1,      /* the kernel records, per ticket, begin/end device time and what its
                           decode of the ticket gave (ft_job_log) */
  FT_PATH_DMA = 1 << 2, /* run the same schedule with hipMemcpyAsync / hipMemcpy2DAsync per
                           chunk piece instead of the copy kernel (comparison path) */
  FT_TIMING = 1 << 3,   /* bracket each class's work with timing events */
  FT_DETACHED = 1 << 4, /* do not make the caller's stream wait for the job */
  FT_KEEP = 1 << 5,     /* keep the job record after ft_wait until ft_job_release;
                           implied by FT_LOG and FT_TIMING */
  FT_OPEN = 1 << 6      /* trigger the chunks in batches and accept ft_submit_merge meanwhile
                           (Sec. 6.1, batched transfer triggering); implies FT_DETACHED; not
                           with FT_PATH_DMA */
};

/*
 * One transfer: rows x row_bytes payload bytes, row r at src + r*src_pitch and
 * dst + r*dst_pitch. Payload order (used by the chunk stream) is row major.
 * After the job completes, for every payload index p with r = p / row_bytes,
 * c = p % row_bytes:   DST[dst + r*dst_pitch + c] == SRC[src + r*src_pitch + c],
 * SRC being memory as it was when the job started (Sec. 5.1: passing is a copy).
 * No alignment is required of src, dst, row_bytes or the pitches.
 */
typedef struct ft_desc {
  uint32_t func;      /* 0 .. nfunc-1: the function this data belongs to */
  uint8_t src_space;  /* FT_HOST: src is a device-visible virtual address of pinned host
                         memory. FT_POOL: src is an ft_off_t. FT_PAGEABLE: a host virtual
                         address inside a window given to ft_pageable_window_add */
  uint8_t dst_space;  /* FT_HOST, FT_POOL or FT_PAGEABLE, as for src. One side must be FT_POOL */
  uint16_t flags;     /* must be 0 */
  uint64_t src;
  uint64_t dst;
  uint64_t row_bytes; /* > 0 */
  uint64_t rows;      /* >= 1; with rows == 1 the pitches are ignored */
  uint64_t src_pitch; /* >= row_bytes when rows > 1 */
  uint64_t dst_pitch; /* >= row_bytes when rows > 1 */
  uint64_t _pad;      /* ignored */
} ft_desc;            /* 64 bytes */

/* Per-class figures of one job (ft_job_stats). */
typedef struct ft_class_stats {
  uint64_t payload_bytes; /* sum of rows*row_bytes of the class's descriptors */
  uint64_t chunks;        /* N = sum over functions of ceil(S_f / chunk_bytes) */
  uint64_t tickets;       /* tiles that hold bytes: what the device counter runs to */
  uint64_t tile_bytes;    /* bytes one ticket moves (last tile of a chunk may be shorter) */
  uint32_t workgroups;    /* persistent workgroups launched (0 on the DMA path) */
  uint32_t in_launch;     /* 1: a small job - tables passed with the launch, run on the caller's stream */
  float device_ms;        /* FT_TIMING: duration of the class's kernel (events bound to its dispatch;
                             on the FT_PATH_DMA path: events around its copy calls), else -1 */
  float begin_ms, end_ms; /* FT_TIMING after ft_timing_epoch: when that kernel began and ended, in ms since
                             the epoch (launches of detached jobs overlap: the time a class was busy is
                             the union of these intervals, not the sum of device_ms), else -1 */
  float _pad2;
} ft_class_stats;

typedef struct ft_job_stats_t {
  ft_class_stats cls[FT_NCLASS];
  double host_submit_us; /* wall time spent inside ft_submit_transfers */
} ft_job_stats_t;

/* ------------------------------------------------------------------ pool (Sec. 7.1) */

/*
 * Create a pool over caller-owned device memory.
 *   out        host pointer, receives the handle.
 *   dev_base   device pointer, 256-byte aligned, valid for `bytes`; must outlive the pool.
 *   bytes      positive multiple of slab_bytes.
 *   slab_bytes positive multiple of 256: the allocation granule.
 *   device     HIP device ordinal the memory lives on.
 * No HIP call is made here. Device resources (one stream per link class, table
 * buffers, events) belong to the device, not the pool: the first ft_submit_transfers
 * on a device creates them, every pool on that device shares them, and they stay
 * until the process ends, so creating and destroying pools is cheap.
 * FT_EINVAL on a null pointer, misalignment or a size that is not a multiple.
 */
int ft_pool_create(ft_pool **out, void *dev_base, uint64_t bytes, uint64_t slab_bytes, int device);

/*
 * Append one segment (the store scales with demand, Sec. 7.1). The logical
 * offset space is the concatenation of the segments in the order added; an
 * allocation never straddles two segments. Same argument rules as create.
 */
int ft_pool_grow(ft_pool *p, void *dev_base, uint64_t bytes);

/* Wait for every job of the pool and free its bookkeeping. Caller memory is untouched. */
int ft_pool_destroy(ft_pool *p);

/*
 * Take the lowest-indexed run of ceil(nbytes / slab_bytes) free slabs that lies in one
 * segment (first fit). *off_out (host pointer) receives its offset.
 * FT_EINVAL if nbytes == 0; FT_ENOMEM if no run exists.
 */
int ft_slab_alloc(ft_pool *p, uint64_t nbytes, ft_off_t *off_out);

/* Return an allocation. FT_EINVAL if off is not the start of a live allocation,
 * FT_EBUSY if a job that has not been waited for refers to it. */
int ft_slab_free(ft_pool *p, ft_off_t off);

/*
 * Give memory back (Sec. 7.1: reserved memory that is no longer needed is reclaimed).
 * Drops the pool's last segment if no allocation lies in it and hands its base and size
 * back to the caller, who owns the memory. FT_EBUSY if an allocation lives there,
 * FT_EINVAL if it is the pool's only segment. First-fit allocation at the lowest offset
 * keeps the late segments empty, so growth and shrinkage are both at the end.
 */
int ft_pool_shrink(ft_pool *p, void **dev_base_out, uint64_t *bytes_out);

/* Bytes of the pool's segments, and bytes of its live allocations (whole slabs). */
int ft_pool_usage(ft_pool *p, uint64_t *total_bytes_out, uint64_t *live_bytes_out);

/* Device pointer of a pool offset, or NULL if off is outside the pool. */
void *ft_pool_ptr(ft_pool *p, ft_off_t off);

/*
 * Declare a window of pinned, device-visible host memory (host pointer that the
 * device can dereference at the same address, e.g. from hipHostMalloc). Once at
 * least one window is registered, every FT_HOST range of a submit must lie inside
 * one window (else FT_ERANGE). With no window registered host ranges are trusted.
 */
int ft_host_window_add(ft_pool *p, void *host_base, uint64_t bytes);

/*
 * Declare a window of ordinary (pageable) host memory that FT_PAGEABLE sources and
 * destinations may lie in; every one must lie inside one (else FT_ERANGE): the library's
 * own threads read and write it. Circular pinned buffer of Sec. 6.1: the device cannot
 * reach such memory, and pinning it call by call or keeping a pinned copy of everything
 * is what the paper rules out, so an open job owns, per direction of the host link in
 * use, one fixed ring of pinned memory, (depth + 1) * batch_chunks slots of one chunk
 * each, shared by all its functions. Host->pool: before a batch is launched the stream
 * bytes of its pageable descriptors are copied into the batch's slots by `threads` host
 * threads (ft_set_batch's neighbour ft_set_stage_threads, default 4) and the copy kernel
 * reads them from there. Pool->host: the kernel writes the batch's slots and the same
 * threads copy them on to the destinations when the batch is complete; ft_wait returns
 * after that. Slots are reused depth + 1 batches later. Source memory must stay valid
 * and unchanged, destination memory valid, until the job has been waited for.
 * A job without FT_OPEN takes a shorter way for little data: if its pageable sides add up
 * to at most 8 MiB (each descriptor rounded up to 16 bytes), ft_submit_transfers copies the
 * pageable sources into a pinned buffer before it returns (they may change afterwards), the
 * device writes pageable destinations into that buffer, and ft_wait copies them on before it
 * returns: only then are they complete, whatever the caller's stream has waited for. More than
 * 8 MiB without FT_OPEN, or FT_PATH_DMA, is FT_EINVAL.
 */
int ft_pageable_window_add(ft_pool *p, void *host_base, uint64_t bytes);

/*
 * Take the pinned memory of the two rings (one per direction of the host link) now, for open
 * jobs of this chunk size under the current ft_set_batch settings, instead of when the first
 * job with pageable memory arrives. A ring's memory stays with the device for the life of the
 * process and serves every later job whose ring fits into it, so this is a call for the start
 * of a long-running process: pinned memory that the runtime hands out early takes device
 * writes faster than memory handed out after other large pinned allocations have come and
 * gone (53 against 46 GB/s towards pageable memory on the machine this was measured on).
 */
int ft_reserve_rings(ft_pool *p, uint64_t chunk_bytes);

/* Host threads (>= 1, the feeder included) that fill the ring of open jobs submitted later. */
int ft_set_stage_threads(ft_pool *p, uint32_t threads);

/* ------------------------------------------------------- transfers (Sec. 5.1, 6.1) */

/*
 * Submit a batch of transfers of nfunc functions.
 *   descs, weights  host pointers; copied before the call returns.
 *   weights[f] >= 1 integer share of function f. chunk_bytes: positive multiple of 16
 *   (the paper's default is 2 MB).
 *   hip_stream      a hipStream_t (NULL = the null stream). The job starts after all work
 *                   already on that stream; unless FT_DETACHED the stream also waits for
 *                   the job, so two jobs on one stream run in submit order. Nothing orders
 *                   two FT_DETACHED jobs with respect to each other: their launches of one
 *                   link class overlap (the head of one fills the compute units that the
 *                   tail of the other leaves idle); a job that reads what a detached job
 *                   writes is submitted after ft_wait for that one.
 *
 * Per link class (host->pool, pool->host, pool->pool) and function, the payloads of
 * the function's descriptors in submission order form a byte stream of S_f bytes;
 * chunk k is stream bytes [k*C, min((k+1)*C, S_f)). All chunks of a class are put in
 * one total order: chunk j of function f carries the finish tag (j+1)/w_f, smaller
 * tags first, equal tags by lower f - i.e. always serve the unfinished function with
 * the smallest (served+1)/weight. Persistent workgroups draw tickets from a device
 * counter in that order; the classes run concurrently on streams of their own.
 * A job of a single link class whose tables fit 3 KiB (not with FT_PATH_DMA,
 * FT_OPEN or a tuned workgroup count) is launched on hip_stream itself with its tables
 * as a kernel argument: same result and order, a tenth of the host time. If it has at
 * most one tile per workgroup (256 tiles pool->pool, 64 host->pool, 128 pool->host) it
 * needs no counter; a larger one takes one of 256 self-clearing counter pairs per device
 * (and the ordinary route if none is free or if FT_DETACHED is set, since the job holds
 * hip_stream like any kernel on it). One contiguous transfer between 16-byte aligned
 * addresses (Sec. 5.1: passing one tensor) needs neither: its tiles are dealt
 * out round robin among the workgroups. Any other job of a single link class without
 * FT_DETACHED also runs on hip_stream itself, its tables copied to the device ahead of it
 * on that stream (the stream was to wait for the job anyway).
 *
 * Validation order: FT_EINVAL conditions of the arguments and of every descriptor
 * (null pointers with non-zero counts, nfunc == 0, a weight of 0, chunk_bytes not a
 * positive multiple of 16, func >= nfunc, flags != 0, a space other than FT_HOST,
 * FT_POOL or FT_PAGEABLE, neither side in the pool, row_bytes == 0, rows == 0, a pitch <
 * row_bytes with rows > 1; more than 8 MiB of FT_PAGEABLE without FT_OPEN is FT_EINVAL after the range checks),
 * then FT_ERANGE of every descriptor, then (FT_VALIDATE) FT_EOVERLAP, and last
 * FT_EINVAL if the weights are so large and so unlike that the schedule tables would
 * exceed 2^22 entries. ndesc == 0 is valid.
 */
int ft_submit_transfers(ft_pool *p, const ft_desc *descs, uint32_t ndesc, const uint32_t *weights,
                        uint32_t nfunc, uint64_t chunk_bytes, uint32_t flags, void *hip_stream,
                        ft_job_t *job_out);

/*
 * Completion (Sec. 8: transfers are asynchronous with function execution, each direction of
 * the host link and the on-device path on streams of their own). ft_submit_transfers only
 * queues work; ft_wait blocks until every chunk of the job is visible at its destination
 * (device memory, and host memory for pool->host). A job can be waited for once; unless it
 * was submitted with FT_KEEP/FT_LOG/FT_TIMING the handle is dead afterwards. The pool's
 * lock is not held while the call blocks: other threads may submit, merge and wait for
 * other jobs of the same pool meanwhile (not destroy the pool).
 */
int ft_wait(ft_pool *p, ft_job_t job);

/* Has everything ft_wait would wait for happened? *done_out (host pointer): 1 or 0. Never blocks;
 * the job still has to be waited for once (which then returns at once). */
int ft_job_done(ft_pool *p, ft_job_t job, int *done_out);

/* Drop the record of a kept job (after ft_wait; FT_EBUSY while a thread is still inside ft_wait for it). */
int ft_job_release(ft_pool *p, ft_job_t job);

/*
 * Sets the instant from which begin_ms / end_ms of ft_job_stats count, for every pool on this
 * pool's device: a timing event recorded on hip_stream and waited for. Call it shortly before the
 * jobs of interest (the times are single-precision milliseconds).
 */
int ft_timing_epoch(ft_pool *p, void *hip_stream);

/* Figures of a kept job (Sec. 8: per-direction streams, so per link class); `out` is a host
 * pointer. device_ms is valid after ft_wait. */
int ft_job_stats(ft_pool *p, ft_job_t job, ft_job_stats_t *out);

/*
 * For callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc. ft_submit_transfers takes table buffers, events and counters from the
 * runtime the first times it runs; this variant takes nothing from it, ever: no hipMalloc, no
 * hipHostMalloc, no event, no stream. The schedule tables and the ticket counter of each link
 * class lie in one array in device memory that is part of the library itself (64 KiB of tables
 * plus one 256-byte counter line per link class, 197 376 bytes on every GPU the library runs on,
 * held until the process ends).
 *   Arguments as for ft_submit_transfers; flags: 0 or FT_VALIDATE. Sides: FT_HOST and FT_POOL only.
 *   Same validation, same chunk order, same copy kernel and tile shapes, same bytes afterwards.
 *   Everything is launched on hip_stream (table pieces travel with small launches, then one copy
 *   kernel per link class in use, one after the other). There is no job handle and nothing to
 *   wait for but the stream: the transfers are complete when the work queued on hip_stream by
 *   this call is. The caller keeps every allocation it names alive until then (no FT_EBUSY
 *   protects them) and may not have two such calls in flight at once on one GPU unless they are
 *   on the same stream: every call on a GPU uses that GPU's one array, so calls that overlap race.
 *   FT_E2BIG, with nothing launched: the tables of some link class do not fit 64 KiB (about 700
 *   descriptors per class; 64-descriptor jobs such as the feature workload take 8 KiB).
 *   FT_EINVAL also for other flags and for FT_PAGEABLE sides (their pinned buffer is an allocation).
 */
int ft_submit_static(ft_pool *p, const ft_desc *descs, uint32_t ndesc, const uint32_t *weights,
                     uint32_t nfunc, uint64_t chunk_bytes, uint32_t flags, void *hip_stream);

/*
 * Batched transfer triggering (Sec. 6.1). A job submitted with FT_OPEN does not hand its
 * whole chunk order to the device at once: per link class a feeder thread launches the
 * copy kernel once per batch of `batch_chunks` consecutive chunks of the order (5 unless
 * ft_set_batch says otherwise) and keeps `depth` batches (3) queued ahead of the device.
 * Transfers merged meanwhile join at the first batch not yet triggered: the order is
 * rebuilt over the chunks not yet triggered of every function already there - each
 * restarting its finish tags at 1/w - plus all chunks of the new functions, functions
 * of earlier jobs before those of later ones in the tie rule, and the following batches
 * come from that order. So a newcomer waits for at most `depth` batches, whatever the
 * length of the jobs before it, and from then on shares the link by weight with them.
 *
 * ft_submit_merge: arguments as ft_submit_transfers; the chunk size is the open job's.
 * The new transfers form a job of their own (own ft_wait, own weights for its nfunc
 * functions, weighed against the other jobs' weights as given). Returns FT_ECLOSED,
 * with nothing merged, if the open job has already triggered its last batch on a link
 * class the new transfers use. Flags: FT_VALIDATE, FT_KEEP (others are taken from the
 * open job). The caller's stream is never made to wait (as with FT_DETACHED); the
 * transfers start after the work already on hip_stream. FT_EINVAL also if open_job is
 * no live handle of a job submitted with FT_OPEN: where merges or weight changes may
 * come after the open job has been waited for, submit it with FT_KEEP, so that they
 * meet FT_ECLOSED (or no effect) rather than a dead handle.
 */
int ft_submit_merge(ft_pool *p, ft_job_t open_job, const ft_desc *descs, uint32_t ndesc,
                    const uint32_t *weights, uint32_t nfunc, uint32_t flags, void *hip_stream,
                    ft_job_t *job_out);

/*
 * Chunks per batch (>= 1) and batches queued ahead (>= 1) for open jobs submitted later.
 * batch_chunks is what a host-link class puts into one batch; the pool->pool class, which
 * moves a chunk some sixty times faster, puts 64 * batch_chunks into one (ft_job_batches
 * reports the batches as triggered).
 */
int ft_set_batch(ft_pool *p, uint32_t batch_chunks, uint32_t depth);

/*
 * Rate control while transfers run (Sec. 6.1: when functions arrive or leave, the idle
 * bandwidth moves to whichever SLO is then the tightest, so the shares of functions
 * already in flight change). Gives the functions of `job` - an open job or one merged
 * into it - new weights, weights[f] >= 1 for each of the nfunc functions the job was
 * submitted with. Batches already triggered are not touched; from the first batch not
 * yet triggered the order is rebuilt over every chunk of the sequence that is left, as
 * for an arrival, with the new weights in force. All or nothing across link classes.
 * batch_out (host, FT_NCLASS entries, may be NULL) receives per link class the number
 * of that first batch, UINT64_MAX where no chunk of the job is left to trigger (the
 * call changes nothing there). The small table upload goes on hip_stream. Thread-safe
 * like ft_submit_merge. FT_EINVAL: unknown job, not part of an open sequence, nfunc
 * differs from the job's, a zero weight.
 */
int ft_job_reweight(ft_pool *p, ft_job_t job, const uint32_t *weights, uint32_t nfunc, void *hip_stream,
                    uint64_t *batch_out);

/*
 * Transfer-rate observation (Sec. 6.1: the rate of each function's data is monitored while it
 * moves, so that it stays above its least rate). For `job` - an open job or one merged into it,
 * whether or not it has been waited for, as long as its record is alive (FT_KEEP) - and one link
 * class: bytes_done[f] (host array of nfunc entries, nfunc as submitted) receives the bytes of
 * function f's chunks whose batch is complete and in place, *batches_done (may be NULL) the
 * number of the sequence's batches seen complete on that class. Two calls a known time apart
 * give every function's rate over that time, at batch grain; a caller that finds a function
 * below its least rate answers with ft_job_reweight. Thread-safe; never blocks on the device.
 * FT_EINVAL: not a job of an open sequence, nfunc differs.
 */
int ft_job_progress(ft_pool *p, ft_job_t job, int link_class, uint64_t *bytes_done, uint32_t nfunc,
                    uint64_t *batches_done);

/*
 * Number of batches of `link_class` that the open job had triggered when `job` joined
 * it (0 for the open job itself): the first batch that may hold the job's chunks.
 */
int ft_job_arrival(ft_pool *p, ft_job_t job, int link_class, uint64_t *batch_out);

/*
 * Test hook: what an open job submitted with FT_KEEP has triggered on `link_class` so
 * far, chunk by chunk in order: the job the chunk belongs to, its function in that job,
 * the chunk's index in the function's stream and the number of the batch. Host arrays
 * of `cap` entries each; *n_out receives the number of chunks triggered.
 */
int ft_job_batches(ft_pool *p, ft_job_t open_job, int link_class, uint64_t *job_out, uint32_t *func_out,
                   uint32_t *chunk_out, uint32_t *batch_out, uint64_t cap, uint64_t *n_out);

/*
 * Function transfer rate control (Sec. 6.1), host-only. For n functions with data sizes
 * (bytes), latency objectives l_slo and inference times l_infer (seconds) on a link of
 * bw_all bytes/s: Rate_least = data_size / (L_slo - L_infer) each; what the link has
 * beyond the sum of the least rates goes to the function with the least time left
 * (lowest index on a tie); nothing is added when the sum already exceeds the link.
 * rate_out (may be NULL) receives the rates, weights_out the integer weights for
 * ft_submit_transfers: each function's share of the rate sum times `total` (0 = 64),
 * rounded half up, at least 1. FT_EINVAL if n == 0, bw_all <= 0 or some L_slo <= L_infer.
 */
int ft_slo_weights(const double *data_size, const double *l_slo, const double *l_infer, uint32_t n,
                   double bw_all, uint32_t total, double *rate_out, uint32_t *weights_out);

/* ------------------------------------------------- elastic data store policies (Sec. 7) */

/*
 * Auto-scaling pool (Sec. 7.1), host only. Per function three histories are kept: the
 * interval between its requests, the size of its intermediate data, and how many of its
 * results are held at once; R_window, R_size, R_con are their `quantile`-th percentiles
 * (nearest rank; 0 = 0.99). ft_sizer_observe(func, t, data_size, concurrency), called
 * after an execution of the function at time t (seconds), reserves R_size * R_con bytes
 * until t + R_window (default_window while the function has been seen only once);
 * ft_sizer_target(t) is the sum of the reservations whose window holds t, at least
 * min_bytes (the paper keeps 300 MB). The caller grows or shrinks the pool to it.
 */
typedef struct ft_sizer ft_sizer;
int ft_sizer_create(ft_sizer **out, uint64_t min_bytes, double quantile, double default_window);
int ft_sizer_observe(ft_sizer *s, uint32_t func, double t, uint64_t data_size, uint32_t concurrency);
int ft_sizer_target(ft_sizer *s, double t, uint64_t *bytes_out);
int ft_sizer_destroy(ft_sizer *s);

/*
 * Queue-aware migration (Sec. 7.2), host only. objs: the stored intermediate data, each
 * with its size, whether it is in GPU memory (resident) and the position in the request
 * queue of the function that will consume it (0 = next). If resident bytes + incoming
 * exceed capacity, evict_ids receives, in order, what to move to host memory until they
 * fit: FT_EVICT_QUEUE_AWARE takes the furthest consumer first (ties: larger id, i.e.
 * stored later); FT_EVICT_LRU, the yardstick, the smallest id first. If nothing has to
 * go, FT_EVICT_QUEUE_AWARE lists in reload_ids what to bring back, nearest consumer
 * first, while it fits entirely. Both arrays hold n entries. The moves themselves are
 * ordinary pool->host and host->pool transfers.
 */
enum { FT_EVICT_QUEUE_AWARE = 0, FT_EVICT_LRU = 1 };
typedef struct ft_object {
  uint64_t id;
  uint64_t bytes;
  uint64_t queue_pos;
  uint32_t resident;
  uint32_t _pad;
} ft_object;
int ft_migrate_plan(const ft_object *objs, uint32_t n, uint64_t capacity, uint64_t incoming, uint32_t policy,
                    uint64_t *evict_ids, uint32_t *n_evict, uint64_t *reload_ids, uint32_t *n_reload);

/*
 * A store of intermediate results under a byte budget, with the queue-aware migration of
 * Sec. 7.2 carried out by the engine itself. `capacity` bytes of results may wait in the
 * pool; `spill_base` / `spill_bytes` is pinned host memory (device-visible, 4096-byte
 * aligned, a multiple of 4096 bytes, owned by the caller; the store declares it to the
 * pool as a host window) that takes what does not fit. ids must grow with store time
 * (ties of the rule go by id); queue_pos is the position of the result's consumer in the
 * request queue (0 = next to run).
 *   ft_store_put      makes room by the rule of ft_migrate_plan (furthest consumer out
 *                     first), allocates nbytes from the pool and returns the offset; the
 *                     caller then writes the result there. FT_ENOMEM: nbytes > capacity,
 *                     the spill arena is full, or the pool has no run of free slabs (grow
 *                     it and call again; what has been moved out stays out). FT_EBUSY: the
 *                     result that would have to leave is still used by a transfer of the
 *                     caller's that has not been waited for; it stays, nothing is stored.
 *   ft_store_get      the consumer runs now: if the result was moved out, room is made
 *                     and it is brought back first (*was_out = 1, host pointer, may be
 *                     NULL). Returns where it is, once it is there: the one call that waits
 *                     for a move, and only for this result's.
 *   ft_store_done     the consumer has finished (and its transfers have been waited for,
 *                     else FT_EBUSY): the result is dropped, and results that were moved
 *                     out come back while they fit, nearest consumer first.
 *   ft_store_advance  the queue has moved: every queue_pos decreases by `steps` (not below 0).
 *   ft_store_sync     waits for every move still in flight (a quiescent point: pool and spill
 *                     arena now hold what the decisions so far imply).
 * Migrations run asynchronously with function execution (Sec. 7.2): every move is one
 * pool->host or host->pool job on hip_stream that put / done / advance do not wait for. The
 * moves pass that stream one after the other, and a slab that a move out has left is handed
 * out again at once, in stream order: the caller writes a result into the offset that put
 * returned with work enqueued on hip_stream (or on a stream that waits for an event recorded on
 * hip_stream after the call), so that the write follows the move that emptied the slabs. The
 * same holds for a consumer that reads a result which is still on its way back without having
 * called ft_store_get for it. Decisions, offsets and bytes are those of carrying out every move
 * at once; only the time at which the bytes are in place differs. One mutex per store.
 */
typedef struct ft_store ft_store;
typedef struct ft_store_stats_t {
  uint64_t objects;        /* results held, in the pool or out */
  uint64_t resident_bytes; /* of them, bytes in the pool */
  uint64_t moved_out, bytes_out;
  uint64_t moved_in, bytes_in;
  uint64_t stalls;         /* ft_store_get calls that had to bring the result back */
  uint64_t moves_in_flight; /* moves nobody has waited for yet */
  uint64_t spill_used_bytes; /* of the spill arena, in whole 4096-byte units */
} ft_store_stats_t;
int ft_store_create(ft_store **out, ft_pool *pool, void *spill_base, uint64_t spill_bytes, uint64_t capacity,
                    uint64_t chunk_bytes, void *hip_stream);
int ft_store_put(ft_store *s, uint64_t id, uint64_t nbytes, uint64_t queue_pos, ft_off_t *off_out);
int ft_store_get(ft_store *s, uint64_t id, ft_off_t *off_out, uint32_t *was_out);
int ft_store_done(ft_store *s, uint64_t id);
int ft_store_advance(ft_store *s, uint64_t steps);
int ft_store_sync(ft_store *s);
int ft_store_stats(ft_store *s, ft_store_stats_t *out);
int ft_store_destroy(ft_store *s);

/* -------------------------------------- parallel paths between GPUs (Sec. 6.2, Alg. 1) */

/*
 * Host-only planner; this library moves no data between GPUs. The server's links are a
 * directed graph: topo[u*n + v] = bandwidth of the link u -> v (0 = none), n <= 16 GPUs.
 * ft_links_select(func, src, dst) chooses parallel paths for a function that sends from
 * src to dst: (1) the loop-free paths from src to dst, fewer hops first and then in
 * lexicographic order of their node sequence, at most max_hops links long (0 = n - 1;
 * at most 4 when n > 8): a path all of whose links are idle is taken, carries the
 * bandwidth of its narrowest link, and that much is subtracted from the free bandwidth of
 * each of its links; this stops when src has no free outgoing or dst no free incoming
 * bandwidth. (2) If both still have some: a busy path is taken over if exactly one path of
 * one other function blocks it, that function holds more bandwidth in total than `func`,
 * and having given the blocking path up it finds an idle path between the same two GPUs
 * that shares no link with the path wanted; it moves there and `func` takes the path.
 * ft_links_paths lists a function's current paths (node sequences back to back in
 * nodes_out, their lengths and bandwidths); ft_links_release gives a function's paths
 * back; ft_links_free copies the n*n matrix of free bandwidth.
 * FT_EINVAL: bad sizes, src == dst, a function that already has paths (select) or has
 * none (paths, release), output arrays too small.
 */
typedef struct ft_links ft_links;
int ft_links_create(ft_links **out, uint32_t n, const uint32_t *topo, uint32_t max_hops);
int ft_links_select(ft_links *l, uint32_t func, uint32_t src, uint32_t dst);
int ft_links_paths(ft_links *l, uint32_t func, uint32_t *nodes_out, uint32_t cap_nodes, uint32_t *len_out,
                   uint32_t *bw_out, uint32_t cap_paths, uint32_t *npaths_out);
int ft_links_release(ft_links *l, uint32_t func);
int ft_links_free(ft_links *l, uint32_t *free_out);
int ft_links_destroy(ft_links *l);

/*
 * Chunks over parallel paths in proportion to the paths' bandwidths (Sec. 6.2): chunk c
 * goes to the path with the smallest (sent + 1) / bandwidth, ties to the lower index -
 * the proportional order of ft_submit_transfers with paths in place of functions.
 */
int ft_stripe_chunks(const uint32_t *path_bw, uint32_t npaths, uint64_t nchunks, uint32_t *path_of_chunk);

/*
 * Test hook: the chunk order of one class of a kept job as a small kernel reads it from the
 * job's tables on the device: every chunk rank is decoded by binary search over the phases
 * (decode_rank, the planner's reference decoder), not by the copy kernel's own cursor-based
 * decode - what that one did ticket by ticket is in the FT_LOG record (ft_job_log).
 * func_out / chunk_out are host arrays of `cap` entries; *n_out receives the number of
 * chunks N (entries beyond cap are not written).
 */
int ft_job_schedule(ft_pool *p, ft_job_t job, int link_class, uint32_t *func_out,
                    uint32_t *chunk_out, uint64_t cap, uint64_t *n_out);

/*
 * FT_LOG: per ticket of one class, after ft_wait, as the copy kernel recorded it: device
 * clock (ns) at claim and at completion, and what the kernel's own decode of the ticket
 * gave - the function, the chunk of the function's stream, the offset of the tile's first
 * byte in that stream and the bytes moved (Sec. 6.1: chunks of different functions are
 * triggered in proportion; this is the order the device really followed). Host arrays of
 * `cap` entries each (any may be NULL); *n_out receives the ticket count.
 */
int ft_job_log(ft_pool *p, ft_job_t job, int link_class, uint64_t *t_begin_ns, uint64_t *t_end_ns,
               uint32_t *func_out, uint32_t *chunk_out, uint64_t *byte_off_out, uint32_t *bytes_out,
               uint64_t cap, uint64_t *n_out);

/*
 * FT_LOG on an open job (ft_job_log then lists every ticket of the whole sequence, merged jobs
 * included, in the order triggered, func_out being the function's index inside its own job):
 * per ticket the job it belongs to and the number of the batch that carried it. Both logs are
 * available once the sequence has run dry on that link class (FT_EBUSY before): wait for the
 * open job and for every job merged into it first. With them the rate of every function can be
 * read off after the fact (Sec. 6.1 monitors it to keep each function above its least rate);
 * ft_job_progress gives the same while the sequence runs, at batch grain.
 */
int ft_job_log_jobs(ft_pool *p, ft_job_t open_job, int link_class, uint64_t *job_out, uint32_t *batch_out,
                    uint64_t cap, uint64_t *n_out);

/*
 * FT_LOG: which workgroup moved each ticket (host array of `cap` entries, may be NULL)
 * and, per workgroup, the device clock (ns) when it started and when it found no
 * ticket left (host arrays of `wg_cap` entries, may be NULL); *nwg_out receives the
 * number of workgroups of the launch. Same clock as ft_job_log. For tuning: shows
 * start-up skew, gaps between tiles and the idle tail of a launch.
 */
int ft_job_log_workgroups(ft_pool *p, ft_job_t job, int link_class, uint32_t *ticket_wg, uint64_t cap,
                          uint64_t *wg_entry_ns, uint64_t *wg_exit_ns, uint32_t wg_cap,
                          uint32_t *nwg_out);

/*
 * FT_LOG: the compute unit every workgroup of the launch ran on (host array of `wg_cap`
 * entries; *nwg_out receives the number of workgroups). The values are identifiers, equal for
 * workgroups that ran on the same unit and otherwise meaningless. Together with the entry and
 * exit times of ft_job_log_workgroups, which share one clock across launches, they show which
 * workgroups of two kernels that ran side by side shared a unit (a job with both host-link
 * and pool->pool traffic runs one kernel per class, Sec. 8: per-direction streams).
 */
int ft_job_log_units(ft_pool *p, ft_job_t job, int link_class, uint32_t *unit_out, uint32_t wg_cap,
                     uint32_t *nwg_out);

/*
 * Launch shape of one class: number of persistent workgroups (0 = default for the
 * device) and bytes per ticket (0 = default; rounded to a multiple of 16 that
 * divides the chunk into equal tiles). Applies to later submits.
 */
int ft_set_tuning(ft_pool *p, int link_class, uint32_t workgroups, uint64_t tile_bytes);

/*
 * Host-only: the chunk order for given per-function stream sizes, computed with
 * the same table builder and rank decoder as the device path, on the CPU. Lets
 * the schedule be checked where no GPU is present. Arrays as in ft_job_schedule.
 */
int ft_plan_schedule(const uint64_t *stream_bytes, const uint32_t *weights, uint32_t nfunc,
                     uint64_t chunk_bytes, uint32_t *func_out, uint32_t *chunk_out, uint64_t cap,
                     uint64_t *n_out);

/*
 * Host-only: the ticket list for given per-function stream sizes and a wanted tile
 * size, computed with the planner's own tile shape, empty-tile runs and ticket
 * mapping. Ticket t moves bytes [byte_off_out[t], byte_off_out[t] + bytes_out[t]) of
 * function func_out[t]'s stream, all inside chunk chunk_out[t]. Host arrays of `cap`
 * entries each; *n_out receives the ticket count. Tickets name only tiles that hold
 * bytes, in the chunk order of ft_plan_schedule, tiles of a chunk in ascending order.
 */
int ft_plan_tickets(const uint64_t *stream_bytes, const uint32_t *weights, uint32_t nfunc,
                    uint64_t chunk_bytes, uint64_t tile_bytes, uint32_t *func_out, uint32_t *chunk_out,
                    uint64_t *byte_off_out, uint32_t *bytes_out, uint64_t cap, uint64_t *n_out);

/*
 * Calibration: a plain grid-stride 16-byte copy of `bytes` (multiple of 16) from
 * src to dst (device pointers, 16-byte aligned) on hip_stream, no tickets, no
 * tables. The practical ceiling the engine is compared with, and the known-size
 * kernel profiler byte counters are scaled by.
 */
int ft_plain_copy(void *dst, const void *src, uint64_t bytes, uint32_t workgroups, void *hip_stream);

/*
 * Calibration: what the memory system gives to reads alone and to writes alone. ft_plain_read
 * loads `bytes` from src and keeps nothing; ft_plain_fill stores `word` over `bytes` at dst
 * (device pointers, 16-byte aligned, bytes a multiple of 16; workgroups 0 = 256). A copy moves
 * every byte once each way, so with read rate R and write rate W it cannot beat
 * 2 / (1/R + 1/W) bytes of traffic per second: the bound `bench.py` reports beside the peak.
 */
int ft_plain_read(const void *src, uint64_t bytes, uint32_t workgroups, void *hip_stream);
int ft_plain_fill(void *dst, uint64_t bytes, uint32_t word, uint32_t workgroups, void *hip_stream);

const char *ft_strerror(int rc);
/* Text of the last failing HIP call on this pool ("" if none). */
const char *ft_last_hip_error(ft_pool *p);

#ifdef __cplusplus
}
#endif
#endif /* FAASTUBE_H */
