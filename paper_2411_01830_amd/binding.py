"""ctypes binding of include/faastube.h: same names, argument marshalling only."""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfaastube.so")

FT_NCLASS = 3
FT_H2P, FT_P2H, FT_P2P = 0, 1, 2
FT_VALIDATE, FT_LOG, FT_PATH_DMA, FT_TIMING, FT_DETACHED, FT_KEEP, FT_OPEN = 1, 2, 4, 8, 16, 32, 64
FT_ECLOSED = -7
FT_E2BIG = -8

EXPORTS = ["ft_pool_create", "ft_pool_grow", "ft_pool_shrink", "ft_pool_usage", "ft_sizer_create",
           "ft_sizer_observe", "ft_sizer_target", "ft_sizer_destroy", "ft_migrate_plan", "ft_links_create",
           "ft_links_select", "ft_links_paths", "ft_links_release", "ft_links_free", "ft_links_destroy",
           "ft_stripe_chunks", "ft_pool_destroy", "ft_slab_alloc", "ft_slab_free",
           "ft_pool_ptr", "ft_store_create", "ft_store_put", "ft_store_get", "ft_store_done", "ft_store_advance", "ft_store_sync", "ft_store_stats", "ft_store_destroy", "ft_host_window_add", "ft_pageable_window_add", "ft_set_stage_threads", "ft_reserve_rings", "ft_submit_transfers", "ft_submit_static", "ft_submit_merge", "ft_job_reweight", "ft_set_batch",
           "ft_job_arrival", "ft_job_batches", "ft_slo_weights", "ft_wait", "ft_job_done", "ft_timing_epoch", "ft_job_release",
           "ft_job_stats", "ft_job_schedule", "ft_job_log", "ft_job_log_jobs", "ft_job_progress", "ft_job_log_workgroups", "ft_job_log_units", "ft_set_tuning", "ft_plan_schedule", "ft_plan_tickets",
           "ft_plain_copy", "ft_plain_read", "ft_plain_fill", "ft_strerror", "ft_last_hip_error"]


class FtError(Exception):
    def __init__(self, code, what=""):
        super().__init__(f"faastube error {code}: {what}")
        self.code = code


class ClassStats(C.Structure):
    _fields_ = [("payload_bytes", C.c_uint64), ("chunks", C.c_uint64), ("tickets", C.c_uint64),
                ("tile_bytes", C.c_uint64), ("workgroups", C.c_uint32), ("in_launch", C.c_uint32),
                ("device_ms", C.c_float), ("begin_ms", C.c_float), ("end_ms", C.c_float), ("_pad2", C.c_float)]


class StoreStats(C.Structure):
    _fields_ = [("objects", C.c_uint64), ("resident_bytes", C.c_uint64), ("moved_out", C.c_uint64),
                ("bytes_out", C.c_uint64), ("moved_in", C.c_uint64), ("bytes_in", C.c_uint64), ("stalls", C.c_uint64), ("moves_in_flight", C.c_uint64), ("spill_used_bytes", C.c_uint64)]


class JobStats(C.Structure):
    _fields_ = [("cls", ClassStats * FT_NCLASS), ("host_submit_us", C.c_double)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python __graft_entry__.py` (or "
                          "paper_2411_01830_amd/build.py) first; there is no CPU fallback")
    # PyTorch ships its own HIP runtime (same SONAME as the system one). The caller's
    # device memory and streams live in that runtime, so it must be the one this library
    # binds to: load it first and the dynamic linker resolves our dependency to it.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, u64, u32, i32 = C.c_void_p, C.c_uint64, C.c_uint32, C.c_int
    P = C.POINTER
    sig = {
        "ft_pool_create": (i32, [P(vp), vp, u64, u64, i32]),
        "ft_pool_grow": (i32, [vp, vp, u64]),
        "ft_pool_destroy": (i32, [vp]),
        "ft_pool_shrink": (i32, [vp, P(vp), P(u64)]),
        "ft_pool_usage": (i32, [vp, P(u64), P(u64)]),
        "ft_sizer_create": (i32, [P(vp), u64, C.c_double, C.c_double]),
        "ft_sizer_observe": (i32, [vp, u32, C.c_double, u64, u32]),
        "ft_sizer_target": (i32, [vp, C.c_double, P(u64)]),
        "ft_sizer_destroy": (i32, [vp]),
        "ft_migrate_plan": (i32, [vp, u32, u64, u64, u32, vp, P(u32), vp, P(u32)]),
        "ft_store_create": (i32, [C.POINTER(vp), vp, vp, u64, u64, u64, vp]),
        "ft_store_put": (i32, [vp, u64, u64, u64, C.POINTER(u64)]),
        "ft_store_get": (i32, [vp, u64, C.POINTER(u64), C.POINTER(u32)]),
        "ft_store_done": (i32, [vp, u64]),
        "ft_store_advance": (i32, [vp, u64]),
        "ft_store_sync": (i32, [vp]),
        "ft_store_stats": (i32, [vp, C.POINTER(StoreStats)]),
        "ft_store_destroy": (i32, [vp]),
        "ft_links_create": (i32, [P(vp), u32, vp, u32]),
        "ft_links_select": (i32, [vp, u32, u32, u32]),
        "ft_links_paths": (i32, [vp, u32, vp, u32, vp, vp, u32, P(u32)]),
        "ft_links_release": (i32, [vp, u32]),
        "ft_links_free": (i32, [vp, vp]),
        "ft_links_destroy": (i32, [vp]),
        "ft_stripe_chunks": (i32, [vp, u32, u64, vp]),
        "ft_slab_alloc": (i32, [vp, u64, P(u64)]),
        "ft_slab_free": (i32, [vp, u64]),
        "ft_pool_ptr": (vp, [vp, u64]),
        "ft_host_window_add": (i32, [vp, vp, u64]),
        "ft_pageable_window_add": (i32, [vp, vp, u64]),
        "ft_set_stage_threads": (i32, [vp, u32]),
        "ft_reserve_rings": (i32, [vp, u64]),
        "ft_submit_transfers": (i32, [vp, vp, u32, vp, u32, u64, u32, vp, P(u64)]),
        "ft_submit_static": (i32, [vp, vp, u32, vp, u32, u64, u32, vp]),
        "ft_submit_merge": (i32, [vp, u64, vp, u32, vp, u32, u32, vp, P(u64)]),
        "ft_job_reweight": (i32, [vp, u64, vp, u32, vp, vp]),
        "ft_set_batch": (i32, [vp, u32, u32]),
        "ft_job_arrival": (i32, [vp, u64, i32, P(u64)]),
        "ft_job_batches": (i32, [vp, u64, i32, vp, vp, vp, vp, u64, P(u64)]),
        "ft_slo_weights": (i32, [vp, vp, vp, u32, C.c_double, u32, vp, vp]),
        "ft_wait": (i32, [vp, u64]),
        "ft_timing_epoch": (i32, [vp, vp]),
        "ft_job_done": (i32, [vp, u64, P(i32)]),
        "ft_job_release": (i32, [vp, u64]),
        "ft_job_stats": (i32, [vp, u64, P(JobStats)]),
        "ft_job_schedule": (i32, [vp, u64, i32, vp, vp, u64, P(u64)]),
        "ft_job_log": (i32, [vp, u64, i32, vp, vp, vp, vp, vp, vp, u64, P(u64)]),
        "ft_job_log_workgroups": (i32, [vp, u64, i32, vp, u64, vp, vp, u32, P(u32)]),
        "ft_job_log_units": (i32, [vp, u64, i32, vp, u32, P(u32)]),
        "ft_job_log_jobs": (i32, [vp, u64, i32, vp, vp, u64, P(u64)]),
        "ft_job_progress": (i32, [vp, u64, i32, vp, u32, P(u64)]),
        "ft_set_tuning": (i32, [vp, i32, u32, u64]),
        "ft_plan_schedule": (i32, [vp, vp, u32, u64, vp, vp, u64, P(u64)]),
        "ft_plan_tickets": (i32, [vp, vp, u32, u64, u64, vp, vp, vp, vp, u64, P(u64)]),
        "ft_plain_copy": (i32, [vp, vp, u64, u32, vp]),
        "ft_plain_read": (i32, [vp, u64, u32, vp]),
        "ft_plain_fill": (i32, [vp, u64, u32, u32, vp]),
        "ft_strerror": (C.c_char_p, [i32]),
        "ft_last_hip_error": (C.c_char_p, [vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


_lib = _load()


def _check(rc, pool=None):
    if rc != 0:
        what = _lib.ft_strerror(rc).decode()
        if rc == -6 and pool:
            what += " - " + _lib.ft_last_hip_error(pool).decode()
        raise FtError(rc, what)


def strerror(rc):
    return _lib.ft_strerror(rc).decode()


def pool_create(dev_base, nbytes, slab_bytes, device=0):
    h = C.c_void_p()
    _check(_lib.ft_pool_create(C.byref(h), dev_base, nbytes, slab_bytes, device))
    return h


def pool_grow(pool, dev_base, nbytes):
    _check(_lib.ft_pool_grow(pool, dev_base, nbytes), pool)


def pool_shrink(pool):
    """(device pointer, bytes) of the segment that was dropped."""
    base, n = C.c_void_p(), C.c_uint64()
    _check(_lib.ft_pool_shrink(pool, C.byref(base), C.byref(n)), pool)
    return base.value, n.value


def pool_usage(pool):
    total, live = C.c_uint64(), C.c_uint64()
    _check(_lib.ft_pool_usage(pool, C.byref(total), C.byref(live)), pool)
    return total.value, live.value


OBJECT_DTYPE = np.dtype([("id", "<u8"), ("bytes", "<u8"), ("queue_pos", "<u8"), ("resident", "<u4"), ("_pad", "<u4")])
FT_EVICT_QUEUE_AWARE, FT_EVICT_LRU = 0, 1


class Sizer:
    """Histogram rule of Sec. 7.1 (ft_sizer_*)."""

    def __init__(self, min_bytes, quantile=0.0, default_window=60.0):
        self._h = C.c_void_p()
        _check(_lib.ft_sizer_create(C.byref(self._h), min_bytes, quantile, default_window))

    def observe(self, func, t, data_size, concurrency):
        _check(_lib.ft_sizer_observe(self._h, func, t, data_size, concurrency))

    def target(self, t):
        out = C.c_uint64()
        _check(_lib.ft_sizer_target(self._h, t, C.byref(out)))
        return out.value

    def close(self):
        if self._h:
            _lib.ft_sizer_destroy(self._h)
            self._h = None


def migrate_plan(objects, capacity, incoming=0, policy=FT_EVICT_QUEUE_AWARE):
    """objects: list of dicts id, bytes, queue_pos, resident -> (evict ids, reload ids)."""
    a = np.zeros(max(len(objects), 1), dtype=OBJECT_DTYPE)
    for i, o in enumerate(objects):
        a[i] = (o["id"], o["bytes"], o["queue_pos"], 1 if o["resident"] else 0, 0)
    ev, rl = np.zeros(len(a), np.uint64), np.zeros(len(a), np.uint64)
    ne, nr = C.c_uint32(), C.c_uint32()
    _check(_lib.ft_migrate_plan(a.ctypes.data, len(objects), capacity, incoming, policy, ev.ctypes.data,
                                C.byref(ne), rl.ctypes.data, C.byref(nr)))
    return ev[:ne.value].tolist(), rl[:nr.value].tolist()


class Store:
    """Store of intermediate results with queue-aware migration (Sec. 7.2; ft_store_*)."""

    def __init__(self, pool, spill_ptr, spill_bytes, capacity, chunk_bytes, stream=None):
        self._h = C.c_void_p()
        self.pool = pool
        _check(_lib.ft_store_create(C.byref(self._h), pool, spill_ptr, spill_bytes, capacity, chunk_bytes, stream), pool)

    def put(self, obj_id, nbytes, queue_pos):
        off = C.c_uint64()
        _check(_lib.ft_store_put(self._h, obj_id, nbytes, queue_pos, C.byref(off)), self.pool)
        return off.value

    def get(self, obj_id):
        off, was_out = C.c_uint64(), C.c_uint32()
        _check(_lib.ft_store_get(self._h, obj_id, C.byref(off), C.byref(was_out)), self.pool)
        return off.value, bool(was_out.value)

    def done(self, obj_id):
        _check(_lib.ft_store_done(self._h, obj_id), self.pool)

    def advance(self, steps):
        _check(_lib.ft_store_advance(self._h, steps), self.pool)

    def sync(self):
        """Wait for every move still in flight (a quiescent point)."""
        _check(_lib.ft_store_sync(self._h), self.pool)

    def stats(self):
        st = StoreStats()
        _check(_lib.ft_store_stats(self._h, C.byref(st)), self.pool)
        return st

    def close(self):
        if self._h:
            _lib.ft_store_destroy(self._h)
            self._h = None


class Links:
    """Path planner of Sec. 6.2 (ft_links_*)."""

    def __init__(self, topo, max_hops=0):
        t = np.ascontiguousarray(np.asarray(topo, dtype=np.uint32))
        self.n = t.shape[0]
        self._h = C.c_void_p()
        _check(_lib.ft_links_create(C.byref(self._h), self.n, t.ctypes.data, max_hops))

    def select(self, func, src, dst):
        _check(_lib.ft_links_select(self._h, func, src, dst))
        return self.paths(func)

    def paths(self, func):
        n = C.c_uint32()
        nodes, ln, bw = np.zeros(4096, np.uint32), np.zeros(256, np.uint32), np.zeros(256, np.uint32)
        _check(_lib.ft_links_paths(self._h, func, nodes.ctypes.data, len(nodes), ln.ctypes.data, bw.ctypes.data,
                                   len(ln), C.byref(n)))
        out, at = [], 0
        for i in range(n.value):
            out.append((tuple(int(x) for x in nodes[at:at + ln[i]]), int(bw[i])))
            at += int(ln[i])
        return out

    def release(self, func):
        _check(_lib.ft_links_release(self._h, func))

    def free(self):
        f = np.zeros(self.n * self.n, np.uint32)
        _check(_lib.ft_links_free(self._h, f.ctypes.data))
        return f.reshape(self.n, self.n).tolist()

    def close(self):
        if self._h:
            _lib.ft_links_destroy(self._h)
            self._h = None


def stripe_chunks(path_bw, nchunks):
    b = np.ascontiguousarray(np.asarray(path_bw, dtype=np.uint32))
    out = np.zeros(max(nchunks, 1), np.uint32)
    _check(_lib.ft_stripe_chunks(b.ctypes.data, len(b), nchunks, out.ctypes.data))
    return out[:nchunks].tolist()


def pool_destroy(pool):
    _check(_lib.ft_pool_destroy(pool))


def slab_alloc(pool, nbytes):
    off = C.c_uint64()
    _check(_lib.ft_slab_alloc(pool, nbytes, C.byref(off)), pool)
    return off.value


def slab_free(pool, off):
    _check(_lib.ft_slab_free(pool, off), pool)


def pool_ptr(pool, off):
    return _lib.ft_pool_ptr(pool, off)


def host_window_add(pool, host_base, nbytes):
    _check(_lib.ft_host_window_add(pool, host_base, nbytes), pool)


class Transfers:
    """Descriptors and weights marshalled once, for a submit that is repeated (a server passing the same
    tensors request after request): the arrays are kept alive here and their addresses are looked up once,
    which is most of what a small submit costs on the Python side. Give it to submit_transfers in place of
    the descriptor array, with weights=None."""
    __slots__ = ("descs", "weights", "d_ptr", "nd", "w_ptr", "nw")

    def __init__(self, descs, weights):
        self.descs = np.ascontiguousarray(descs)
        assert self.descs.dtype.itemsize == 64
        self.weights = np.ascontiguousarray(np.asarray(weights, dtype=np.uint32))
        self.nd, self.nw = len(self.descs), len(self.weights)
        self.d_ptr = self.descs.ctypes.data if self.nd else None
        self.w_ptr = self.weights.ctypes.data if self.nw else None


def submit_transfers(pool, descs, weights, chunk_bytes, flags=0, stream=0):
    """descs: contiguous array of the 64-byte descriptor dtype; weights: uint32 sequence. Or descs: a
    Transfers object (then weights is None)."""
    if isinstance(descs, Transfers):
        job = C.c_uint64()
        _check(_lib.ft_submit_transfers(pool, descs.d_ptr, descs.nd, descs.w_ptr, descs.nw, chunk_bytes, flags,
                                        stream, C.byref(job)), pool)
        return job.value
    if not descs.flags.c_contiguous:
        descs = np.ascontiguousarray(descs)
    assert descs.dtype.itemsize == 64
    w = weights if isinstance(weights, np.ndarray) and weights.dtype == np.uint32 and weights.flags.c_contiguous \
        else np.ascontiguousarray(np.asarray(weights, dtype=np.uint32))
    job = C.c_uint64()
    _check(_lib.ft_submit_transfers(pool, descs.ctypes.data if len(descs) else None, len(descs),
                                    w.ctypes.data if len(w) else None, len(w), chunk_bytes, flags,
                                    stream, C.byref(job)), pool)
    return job.value


def submit_static(pool, descs, weights, chunk_bytes, flags=0, stream=0):
    """ft_submit_static: the submit that allocates nothing; complete when the stream has passed it."""
    descs = np.ascontiguousarray(descs)
    assert descs.dtype.itemsize == 64
    w = np.ascontiguousarray(np.asarray(weights, dtype=np.uint32))
    _check(_lib.ft_submit_static(pool, descs.ctypes.data if len(descs) else None, len(descs),
                                 w.ctypes.data if len(w) else None, len(w), chunk_bytes, flags, stream), pool)


def wait(pool, job):
    _check(_lib.ft_wait(pool, job), pool)


def job_done(pool, job):
    d = C.c_int()
    _check(_lib.ft_job_done(pool, job, C.byref(d)), pool)
    return bool(d.value)


def timing_epoch(pool, stream=0):
    _check(_lib.ft_timing_epoch(pool, stream), pool)


def job_release(pool, job):
    _check(_lib.ft_job_release(pool, job), pool)


def job_stats(pool, job):
    st = JobStats()
    _check(_lib.ft_job_stats(pool, job, C.byref(st)), pool)
    return st


def job_schedule(pool, job, link_class):
    n = C.c_uint64()
    _check(_lib.ft_job_schedule(pool, job, link_class, None, None, 0, C.byref(n)), pool)
    f = np.zeros(max(n.value, 1), dtype=np.uint32)
    k = np.zeros(max(n.value, 1), dtype=np.uint32)
    _check(_lib.ft_job_schedule(pool, job, link_class, f.ctypes.data, k.ctypes.data, n.value,
                                C.byref(n)), pool)
    return list(zip(f[:n.value].tolist(), k[:n.value].tolist()))


def job_log(pool, job, link_class):
    """dict of arrays, one entry per ticket, all of it recorded by the copy kernel: t_begin_ns,
    t_end_ns, and the kernel's own decode of the ticket: func, chunk, byte_off, bytes."""
    n = C.c_uint64()
    _check(_lib.ft_job_log(pool, job, link_class, None, None, None, None, None, None, 0, C.byref(n)), pool)
    m = max(n.value, 1)
    tb, te, bo = np.zeros(m, np.uint64), np.zeros(m, np.uint64), np.zeros(m, np.uint64)
    f, k, b = np.zeros(m, np.uint32), np.zeros(m, np.uint32), np.zeros(m, np.uint32)
    _check(_lib.ft_job_log(pool, job, link_class, tb.ctypes.data, te.ctypes.data, f.ctypes.data,
                           k.ctypes.data, bo.ctypes.data, b.ctypes.data, n.value, C.byref(n)), pool)
    s = slice(0, n.value)
    return {"t_begin_ns": tb[s], "t_end_ns": te[s], "func": f[s], "chunk": k[s], "byte_off": bo[s], "bytes": b[s]}


def job_log_jobs(pool, open_job, link_class):
    """FT_LOG on an open job: per ticket of the sequence (parallel to job_log) the job id and the batch."""
    n = C.c_uint64()
    _check(_lib.ft_job_log_jobs(pool, open_job, link_class, None, None, 0, C.byref(n)), pool)
    m = max(n.value, 1)
    j, b = np.zeros(m, np.uint64), np.zeros(m, np.uint32)
    _check(_lib.ft_job_log_jobs(pool, open_job, link_class, j.ctypes.data, b.ctypes.data, n.value, C.byref(n)), pool)
    return {"job": j[:n.value], "batch": b[:n.value]}


def job_progress(pool, job, link_class, nfunc):
    """(bytes complete per function of the job, batches of the sequence complete) on one link class."""
    done, nb = np.zeros(max(nfunc, 1), np.uint64), C.c_uint64()
    _check(_lib.ft_job_progress(pool, job, link_class, done.ctypes.data, nfunc, C.byref(nb)), pool)
    return done[:nfunc].tolist(), nb.value


def job_log_workgroups(pool, job, link_class, ntickets):
    """(workgroup of each ticket, entry ns per workgroup, exit ns per workgroup)."""
    nwg = C.c_uint32()
    _check(_lib.ft_job_log_workgroups(pool, job, link_class, None, 0, None, None, 0, C.byref(nwg)), pool)
    wg = np.zeros(max(int(ntickets), 1), np.uint32)
    t_in, t_out = np.zeros(max(nwg.value, 1), np.uint64), np.zeros(max(nwg.value, 1), np.uint64)
    _check(_lib.ft_job_log_workgroups(pool, job, link_class, wg.ctypes.data, int(ntickets), t_in.ctypes.data,
                                      t_out.ctypes.data, nwg.value, C.byref(nwg)), pool)
    return wg[:int(ntickets)], t_in[:nwg.value], t_out[:nwg.value]


def job_log_units(pool, job, link_class):
    """Identifier of the compute unit each workgroup of the launch ran on."""
    nwg = C.c_uint32()
    _check(_lib.ft_job_log_units(pool, job, link_class, None, 0, C.byref(nwg)), pool)
    unit = np.zeros(max(nwg.value, 1), np.uint32)
    _check(_lib.ft_job_log_units(pool, job, link_class, unit.ctypes.data, nwg.value, C.byref(nwg)), pool)
    return unit[:nwg.value]


def set_tuning(pool, link_class, workgroups=0, tile_bytes=0):
    _check(_lib.ft_set_tuning(pool, link_class, workgroups, tile_bytes), pool)


def plan_schedule(stream_bytes, weights, chunk_bytes):
    s = np.ascontiguousarray(np.asarray(stream_bytes, dtype=np.uint64))
    w = np.ascontiguousarray(np.asarray(weights, dtype=np.uint32))
    n = C.c_uint64()
    _check(_lib.ft_plan_schedule(s.ctypes.data, w.ctypes.data, len(w), chunk_bytes, None, None, 0,
                                 C.byref(n)))
    f = np.zeros(max(n.value, 1), dtype=np.uint32)
    k = np.zeros(max(n.value, 1), dtype=np.uint32)
    _check(_lib.ft_plan_schedule(s.ctypes.data, w.ctypes.data, len(w), chunk_bytes, f.ctypes.data,
                                 k.ctypes.data, n.value, C.byref(n)))
    return list(zip(f[:n.value].tolist(), k[:n.value].tolist()))


def submit_merge(pool, open_job, descs, weights, flags=0, stream=0):
    d = np.ascontiguousarray(descs)
    w = np.ascontiguousarray(np.asarray(weights, dtype=np.uint32))
    job = C.c_uint64()
    _check(_lib.ft_submit_merge(pool, open_job, d.ctypes.data, len(d), w.ctypes.data, len(w), flags, stream,
                                C.byref(job)), pool)
    return job.value


def job_reweight(pool, job, weights, stream=0):
    """New weights for the job's functions; per link class the first batch they hold for (None: none left)."""
    w = np.ascontiguousarray(np.asarray(weights, dtype=np.uint32))
    b = (C.c_uint64 * 3)()
    _check(_lib.ft_job_reweight(pool, job, w.ctypes.data, len(w), stream, C.cast(b, C.c_void_p)), pool)
    return [None if v == 2 ** 64 - 1 else int(v) for v in b]


def pageable_window_add(pool, host_ptr, nbytes):
    _check(_lib.ft_pageable_window_add(pool, host_ptr, nbytes), pool)


def reserve_rings(pool, chunk_bytes):
    _check(_lib.ft_reserve_rings(pool, chunk_bytes), pool)


def set_stage_threads(pool, threads):
    _check(_lib.ft_set_stage_threads(pool, threads), pool)


def set_batch(pool, batch_chunks=5, depth=2):
    _check(_lib.ft_set_batch(pool, batch_chunks, depth), pool)


def job_arrival(pool, job, link_class):
    b = C.c_uint64()
    _check(_lib.ft_job_arrival(pool, job, link_class, C.byref(b)), pool)
    return b.value


def job_batches(pool, open_job, link_class):
    """List of batches; a batch is a list of (job handle, function, chunk)."""
    n = C.c_uint64()
    _check(_lib.ft_job_batches(pool, open_job, link_class, None, None, None, None, 0, C.byref(n)), pool)
    m = max(n.value, 1)
    j, f, k, b = np.zeros(m, np.uint64), np.zeros(m, np.uint32), np.zeros(m, np.uint32), np.zeros(m, np.uint32)
    _check(_lib.ft_job_batches(pool, open_job, link_class, j.ctypes.data, f.ctypes.data, k.ctypes.data,
                               b.ctypes.data, n.value, C.byref(n)), pool)
    out = []
    for i in range(min(n.value, m)):
        while len(out) <= int(b[i]):
            out.append([])
        out[int(b[i])].append((int(j[i]), int(f[i]), int(k[i])))
    return out


def slo_weights(data_size, l_slo, l_infer, bw_all, total=0):
    """(rates, weights) of Sec. 6.1's transfer rate control."""
    a = [np.ascontiguousarray(np.asarray(x, dtype=np.float64)) for x in (data_size, l_slo, l_infer)]
    n = len(a[0])
    rate, w = np.zeros(max(n, 1), np.float64), np.zeros(max(n, 1), np.uint32)
    _check(_lib.ft_slo_weights(a[0].ctypes.data, a[1].ctypes.data, a[2].ctypes.data, n, float(bw_all), total,
                               rate.ctypes.data, w.ctypes.data))
    return rate[:n].tolist(), w[:n].tolist()


def plan_tickets(stream_bytes, weights, chunk_bytes, tile_bytes):
    """List of (func, chunk, byte offset in the function's stream, bytes), one per ticket."""
    s = np.ascontiguousarray(np.asarray(stream_bytes, dtype=np.uint64))
    w = np.ascontiguousarray(np.asarray(weights, dtype=np.uint32))
    n = C.c_uint64()
    _check(_lib.ft_plan_tickets(s.ctypes.data, w.ctypes.data, len(w), chunk_bytes, tile_bytes, None, None,
                                None, None, 0, C.byref(n)))
    m = max(n.value, 1)
    f, k = np.zeros(m, np.uint32), np.zeros(m, np.uint32)
    off, b = np.zeros(m, np.uint64), np.zeros(m, np.uint32)
    _check(_lib.ft_plan_tickets(s.ctypes.data, w.ctypes.data, len(w), chunk_bytes, tile_bytes, f.ctypes.data,
                                k.ctypes.data, off.ctypes.data, b.ctypes.data, n.value, C.byref(n)))
    q = slice(0, n.value)
    return list(zip(f[q].tolist(), k[q].tolist(), off[q].tolist(), b[q].tolist()))


def plain_copy(dst_ptr, src_ptr, nbytes, workgroups=0, stream=0):
    _check(_lib.ft_plain_copy(dst_ptr, src_ptr, nbytes, workgroups, stream))


def plain_read(src_ptr, nbytes, workgroups=0, stream=0):
    _check(_lib.ft_plain_read(src_ptr, nbytes, workgroups, stream))


def plain_fill(dst_ptr, nbytes, word, workgroups=0, stream=0):
    _check(_lib.ft_plain_fill(dst_ptr, nbytes, word, workgroups, stream))
