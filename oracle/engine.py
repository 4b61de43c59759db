"""The engine calls on host memory: validation, overlap check, byte movement.

Sec. 5.1: passing data between host and GPU memory, and between two functions
on one GPU, is a copy; chunking (Sec. 6.1) only decides the order in which
pieces travel. So after a job completes, for every descriptor d and payload
index p, with r = p div row_bytes and c = p mod row_bytes,

    DST[d.dst + r * d.dst_pitch + c] = SRC[d.src + r * d.src_pitch + c]

and every other byte keeps its value. ``submit`` below moves the bytes chunk
by chunk in ticket order (the algorithm); ``apply_definition`` writes the
same result straight from the formula. The tests hold one against the other.

Host memory is modelled as one flat array (addresses are offsets into it),
the pool as one flat array over its logical offset space.
"""
import numpy as np

from . import (OracleError, EINVAL, ERANGE, EOVERLAP, EBUSY, HOST, POOL, PAGEABLE,
               H2P, P2H, P2P)
from .pool import Pool
from .schedule import link_class, chunk_count, stride_order, chunk_segments

U32_MAX = (1 << 32) - 1
U64_MAX = (1 << 64) - 1


def _extent(row_bytes, rows, pitch):
    return (rows - 1) * pitch + row_bytes


def _row_intervals(descs, which, space):
    """Sorted [start, end) of every row, on the src or dst side, that lies in `space`."""
    starts = []
    ends = []
    for d in descs:
        if int(d[which + "_space"]) != space:
            continue
        rows = int(d["rows"])
        s = int(d[which]) + np.arange(rows, dtype=np.int64) * (int(d[which + "_pitch"]) if rows > 1 else 0)
        starts.append(s)
        ends.append(s + int(d["row_bytes"]))
    if not starts:
        return np.zeros(0, np.int64), np.zeros(0, np.int64)
    starts = np.concatenate(starts)
    ends = np.concatenate(ends)
    order = np.argsort(starts, kind="stable")
    return starts[order], ends[order]


def find_overlap(descs):
    """True if some destination byte is also a destination byte of another
    row/descriptor, or a source byte, of the same submit (same address space).

    Disjoint destinations make the result independent of the order in which
    chunks complete; that is why aliasing is rejected."""
    for space in (HOST, POOL, PAGEABLE):
        d0, d1 = _row_intervals(descs, "dst", space)
        if len(d0) == 0:
            continue
        # destinations sorted by start: pairwise disjoint iff each ends before the next starts
        if np.any(d0[1:] < d1[:-1]):
            return True
        s0, s1 = _row_intervals(descs, "src", space)
        if len(s0) == 0:
            continue
        # destinations are now disjoint, so their ends are sorted too: the only
        # candidate for a source row is the first destination ending after its start
        idx = np.searchsorted(d1, s0, side="right")
        ok = idx < len(d0)
        if np.any(d0[idx[ok]] < s1[ok]):
            return True
    return False


class _Job:
    def __init__(self, jid):
        self.id = jid
        self.pending = True
        self.allocs = set()
        self.schedule = {H2P: [], P2H: [], P2P: []}
        self.class_bytes = {H2P: 0, P2H: 0, P2P: 0}


class OracleEngine:
    """Same calls as the C library, on host arrays."""

    def __init__(self):
        self.pool = None
        self.pool_mem = None
        self.host_mem = np.zeros(0, dtype=np.uint8)
        self.pageable_mem = np.zeros(0, dtype=np.uint8)
        self.jobs = {}
        self._next_job = 1

    # ---- memory the caller owns -------------------------------------------------
    def host_arena(self, nbytes, fill=0x5A):
        self.host_mem = np.full(nbytes, fill, dtype=np.uint8)

    def pageable_arena(self, nbytes, fill=0x3C):
        """Ordinary host memory (the host side of a transfer). Addresses are offsets into it."""
        self.pageable_mem = np.full(nbytes, fill, dtype=np.uint8)

    def write_pageable(self, off, data):
        self.pageable_mem[off:off + len(data)] = data

    def write_host(self, off, data):
        self.host_mem[off:off + len(data)] = data

    def read_host(self, off, n):
        return self.host_mem[off:off + n].copy()

    def write_pool(self, off, data):
        self.pool_mem[off:off + len(data)] = data

    def read_pool(self, off, n):
        return self.pool_mem[off:off + n].copy()

    # ---- pool -------------------------------------------------------------------
    def pool_create(self, nbytes, slab_bytes, fill=0xA5):
        self.pool = Pool(nbytes, slab_bytes)
        self.pool_mem = np.full(nbytes, fill, dtype=np.uint8)
        self._fill = fill

    def pool_grow(self, nbytes):
        self.pool.grow(nbytes)
        self.pool_mem = np.concatenate(
            [self.pool_mem, np.full(nbytes, self._fill, dtype=np.uint8)])

    def pool_shrink(self):
        n = self.pool.shrink()
        self.pool_mem = self.pool_mem[:len(self.pool_mem) - n].copy()
        return n

    def slab_alloc(self, nbytes):
        return self.pool.alloc(nbytes)

    def slab_free(self, off):
        for job in self.jobs.values():
            if job.pending and off in job.allocs:
                raise OracleError(EBUSY, "allocation is referenced by a job not yet waited for")
        self.pool.free(off)

    # ---- transfers --------------------------------------------------------------
    def _check(self, descs, weights, chunk_bytes):
        nfunc = len(weights)
        if nfunc < 1:
            raise OracleError(EINVAL, "no functions")
        for w in weights:
            if int(w) < 1 or int(w) > U32_MAX:
                raise OracleError(EINVAL, "weight must be >= 1")
        if chunk_bytes <= 0 or chunk_bytes % 16 != 0:
            raise OracleError(EINVAL, "chunk_bytes must be a positive multiple of 16")
        for d in descs:
            if int(d["func"]) >= nfunc or int(d["flags"]) != 0:
                raise OracleError(EINVAL, "bad func or flags")
            if int(d["src_space"]) not in (HOST, POOL, PAGEABLE) or int(d["dst_space"]) not in (HOST, POOL, PAGEABLE):
                raise OracleError(EINVAL, "bad space")
            link_class(int(d["src_space"]), int(d["dst_space"]))
            if int(d["row_bytes"]) == 0 or int(d["rows"]) == 0:
                raise OracleError(EINVAL, "empty descriptor")
            if int(d["rows"]) > 1 and (int(d["src_pitch"]) < int(d["row_bytes"])
                                       or int(d["dst_pitch"]) < int(d["row_bytes"])):
                raise OracleError(EINVAL, "pitch smaller than a row")
        used = set()
        for d in descs:
            for side in ("src", "dst"):
                off = int(d[side])
                ext = _extent(int(d["row_bytes"]), int(d["rows"]),
                              int(d[side + "_pitch"]) if int(d["rows"]) > 1 else 0)
                if off + ext > U64_MAX:
                    raise OracleError(ERANGE, "range wraps")
                if int(d[side + "_space"]) == POOL:
                    a = self.pool.owner(off, ext) if self.pool is not None else None
                    if a is None:
                        raise OracleError(ERANGE, "pool range not inside one live allocation")
                    used.add(a)
                elif int(d[side + "_space"]) == PAGEABLE:
                    if off + ext > len(self.pageable_mem):
                        raise OracleError(ERANGE, "pageable range outside its window")
                else:
                    if off + ext > len(self.host_mem):
                        raise OracleError(ERANGE, "host range outside the arena")
        if find_overlap(descs):
            raise OracleError(EOVERLAP, "a destination byte is written twice or also read")
        return used

    def _mem(self, space):
        return self.host_mem if space == HOST else self.pageable_mem if space == PAGEABLE else self.pool_mem

    def submit(self, descs, weights, chunk_bytes, flags=0):
        used = self._check(descs, weights, chunk_bytes)
        job = _Job(self._next_job)
        self._next_job += 1
        job.allocs = used
        nfunc = len(weights)
        for cls in (H2P, P2H, P2P):
            mine = [d for d in descs
                    if link_class(int(d["src_space"]), int(d["dst_space"])) == cls]
            per_func = [[d for d in mine if int(d["func"]) == f] for f in range(nfunc)]
            stream = [sum(int(d["row_bytes"]) * int(d["rows"]) for d in ds) for ds in per_func]
            n = [chunk_count(s, chunk_bytes) for s in stream]
            order = stride_order(n, [int(w) for w in weights])
            job.schedule[cls] = order
            job.class_bytes[cls] = sum(stream)
            for f, k in order:
                ds = per_func[f]
                shape = [(int(d["row_bytes"]), int(d["rows"])) for d in ds]
                for di, r, c, length in chunk_segments(shape, chunk_bytes, k):
                    d = ds[di]
                    s = int(d["src"]) + r * int(d["src_pitch"]) + c
                    t = int(d["dst"]) + r * int(d["dst_pitch"]) + c
                    self._mem(int(d["dst_space"]))[t:t + length] = \
                        self._mem(int(d["src_space"]))[s:s + length]
        self.jobs[job.id] = job
        return job.id

    def apply_definition(self, descs):
        """The data result written straight from the formula, no chunks."""
        for d in descs:
            src = self._mem(int(d["src_space"]))
            dst = self._mem(int(d["dst_space"]))
            rb = int(d["row_bytes"])
            for r in range(int(d["rows"])):
                s = int(d["src"]) + r * int(d["src_pitch"])
                t = int(d["dst"]) + r * int(d["dst_pitch"])
                dst[t:t + rb] = src[s:s + rb]

    def wait(self, job_id):
        job = self.jobs.get(job_id)
        if job is None or not job.pending:
            raise OracleError(EINVAL, "no such pending job")
        job.pending = False

    def job_schedule(self, job_id, cls):
        return list(self.jobs[job_id].schedule[cls])

    def job_class_bytes(self, job_id, cls):
        return self.jobs[job_id].class_bytes[cls]
