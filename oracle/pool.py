"""Slab pool of the GPU store (Sec. 7.1), as plain bookkeeping.

The paper keeps intermediate data in a pool of GPU memory blocks so that data
passing never pays for native allocation, and lets the pool scale with
demand. It gives no allocation algorithm. Reading taken here: the pool is an
ordered list of segments, its logical byte-offset space is their
concatenation, a request takes the lowest-indexed run of free slabs that is
long enough and lies inside one segment (first fit), growth appends a
segment, and the pool gives memory back (Sec. 7.1: reserved memory that is no
longer needed is reclaimed) by dropping its last segment when nothing lives in
it - never the first one.
"""
from . import OracleError, EINVAL, ENOMEM, EBUSY


class Pool:
    def __init__(self, nbytes, slab_bytes):
        if slab_bytes <= 0 or slab_bytes % 256 != 0:
            raise OracleError(EINVAL, "slab_bytes must be a positive multiple of 256")
        if nbytes <= 0 or nbytes % slab_bytes != 0:
            raise OracleError(EINVAL, "segment must be a positive multiple of slab_bytes")
        self.slab_bytes = slab_bytes
        self.segments = []        # (first_slab, nslabs) in growth order
        self.used = []            # one flag per slab
        self.allocs = {}          # offset -> number of slabs
        self._append(nbytes)

    def _append(self, nbytes):
        n = nbytes // self.slab_bytes
        self.segments.append((len(self.used), n))
        self.used.extend([False] * n)

    @property
    def total_bytes(self):
        return len(self.used) * self.slab_bytes

    def grow(self, nbytes):
        if nbytes <= 0 or nbytes % self.slab_bytes != 0:
            raise OracleError(EINVAL, "segment must be a positive multiple of slab_bytes")
        self._append(nbytes)

    def shrink(self):
        """Drop the last segment; returns its size in bytes."""
        if len(self.segments) < 2:
            raise OracleError(EINVAL, "the first segment stays")
        first, n = self.segments[-1]
        if any(self.used[first:first + n]):
            raise OracleError(EBUSY, "an allocation lives in the last segment")
        self.segments.pop()
        del self.used[first:]
        return n * self.slab_bytes

    @property
    def live_bytes(self):
        return sum(self.allocs.values()) * self.slab_bytes

    def alloc(self, nbytes):
        if nbytes <= 0:
            raise OracleError(EINVAL, "nbytes must be positive")
        need = -(-nbytes // self.slab_bytes)
        for first, n in self.segments:
            for start in range(first, first + n - need + 1):
                if not any(self.used[start:start + need]):
                    for i in range(start, start + need):
                        self.used[i] = True
                    off = start * self.slab_bytes
                    self.allocs[off] = need
                    return off
        raise OracleError(ENOMEM, "no run of free slabs")

    def free(self, off):
        if off not in self.allocs:
            raise OracleError(EINVAL, "not the start of a live allocation")
        need = self.allocs.pop(off)
        start = off // self.slab_bytes
        for i in range(start, start + need):
            self.used[i] = False

    def owner(self, off, extent):
        """Start offset of the live allocation that holds [off, off+extent), else None."""
        for a, need in self.allocs.items():
            if a <= off and off + extent <= a + need * self.slab_bytes:
                return a
        return None
