"""Device and pinned memory for the engine, owned through PyTorch.

``GpuEngine`` exposes the engine calls in the shape the workload runner expects
(host addresses are offsets into one pinned arena; the pool's segments are uint8
device tensors). PyTorch is used for memory, streams and read-back only; every
transfer goes through the C ABI.
"""
import numpy as np
import torch

from . import binding as ft

HOST_FILL = 0x5A
POOL_FILL = 0xA5


class GpuEngine:
    def __init__(self, device=0, register_window=True, reuse_memory=False):
        if not torch.cuda.is_available():
            raise RuntimeError("GpuEngine needs a GPU; the engine has no CPU path")
        self.device = device
        self.dev = torch.device("cuda", device)
        self.pool = None
        self.segments = []          # (tensor, logical first byte)
        self.total = 0
        self.host = None
        self.host_np = None
        self.pageable_np = None
        self.register_window = register_window
        self.default_flags = 0
        # reuse_memory: device segments and the pinned arena survive close_pool() and are
        # handed out again, in the same order, to the next pool_create / pool_grow, so a
        # benchmark step pays for the engine's work and not for hipMalloc
        self.reuse_memory = reuse_memory
        self._seg_cache = []
        self._seg_next = 0

    # ---- caller-owned memory ---------------------------------------------------
    def host_arena(self, nbytes, fill=HOST_FILL):
        nbytes = max(int(nbytes), 4096)
        if self.reuse_memory and self.host is not None and self.host.numel() == nbytes:
            pass
        else:
            self.host = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
            self.host_np = self.host.numpy()
            if fill is not None:
                self.host_np[:] = fill
        if self.pool is not None and self.register_window:
            ft.host_window_add(self.pool, self.host.data_ptr(), nbytes)

    def pageable_arena(self, nbytes, fill=0x3C):
        """Ordinary (not pinned) host memory for FT_PAGEABLE; addresses are offsets into it."""
        # anonymous memory that the kernel may back with huge pages, as a long-lived process's heap would be
        import mmap
        self._pageable_map = mmap.mmap(-1, int(nbytes))
        if hasattr(mmap, "MADV_HUGEPAGE"):
            try:
                self._pageable_map.madvise(mmap.MADV_HUGEPAGE)
            except OSError:
                pass
        self.pageable_np = np.frombuffer(self._pageable_map, dtype=np.uint8)
        self.pageable_np[:] = fill
        if self.pool is not None:
            ft.pageable_window_add(self.pool, self.pageable_np.ctypes.data, int(nbytes))

    def write_pageable(self, off, data):
        self.pageable_np[off:off + len(data)] = data

    def write_host(self, off, data):
        self.host_np[off:off + len(data)] = data

    def read_host(self, off, n):
        return self.host_np[off:off + n].copy()

    def _segment(self, nbytes, fill):
        if self.reuse_memory and self._seg_next < len(self._seg_cache) and \
                self._seg_cache[self._seg_next].numel() == int(nbytes):
            t = self._seg_cache[self._seg_next]
            self._seg_next += 1
            return t
        t = torch.empty(int(nbytes), dtype=torch.uint8, device=self.dev)
        if fill is not None:
            t.fill_(fill)
        if self.reuse_memory:
            del self._seg_cache[self._seg_next:]
            self._seg_cache.append(t)
            self._seg_next += 1
        assert t.data_ptr() % 256 == 0
        return t

    def _locate(self, off):
        for t, first in self.segments:
            if first <= off < first + t.numel():
                return t, off - first
        raise IndexError(off)

    def write_pool(self, off, data):
        t, o = self._locate(off)
        t[o:o + len(data)].copy_(torch.from_numpy(np.ascontiguousarray(data)))

    def read_pool(self, off, n):
        t, o = self._locate(off)
        return t[o:o + n].cpu().numpy()

    # ---- pool --------------------------------------------------------------------
    def pool_create(self, nbytes, slab_bytes, fill=POOL_FILL):
        t = self._segment(nbytes, fill)
        self._fill = fill
        self.pool = ft.pool_create(t.data_ptr(), int(nbytes), int(slab_bytes), self.device)
        self.segments = [(t, 0)]
        self.total = int(nbytes)
        if self.host is not None and self.register_window:
            ft.host_window_add(self.pool, self.host.data_ptr(), self.host.numel())
        if self.pageable_np is not None:
            ft.pageable_window_add(self.pool, self.pageable_np.ctypes.data, len(self.pageable_np))

    def pool_grow(self, nbytes):
        t = self._segment(nbytes, self._fill)
        ft.pool_grow(self.pool, t.data_ptr(), int(nbytes))
        self.segments.append((t, self.total))
        self.total += int(nbytes)

    def slab_alloc(self, nbytes):
        return ft.slab_alloc(self.pool, int(nbytes))

    def slab_free(self, off):
        ft.slab_free(self.pool, int(off))

    # ---- transfers ---------------------------------------------------------------
    def submit(self, descs, weights, chunk_bytes, flags=0, stream=None):
        d = np.array(descs, copy=True)
        base = self.host.data_ptr() if self.host is not None else 0
        d["src"][d["src_space"] == 0] += np.uint64(base)
        d["dst"][d["dst_space"] == 0] += np.uint64(base)
        if np.any(d["src_space"] == 2):
            d["src"][d["src_space"] == 2] += np.uint64(self.pageable_np.ctypes.data)
        if np.any(d["dst_space"] == 2):
            d["dst"][d["dst_space"] == 2] += np.uint64(self.pageable_np.ctypes.data)
        s = torch.cuda.current_stream(self.dev).cuda_stream if stream is None else stream
        return ft.submit_transfers(self.pool, d, weights, int(chunk_bytes),
                                   int(flags) | self.default_flags, s)

    def submit_static(self, descs, weights, chunk_bytes, flags=0, stream=None):
        """ft_submit_static on the current (or given) stream; complete when that stream is."""
        d = np.array(descs, copy=True)
        base = self.host.data_ptr() if self.host is not None else 0
        d["src"][d["src_space"] == 0] += np.uint64(base)
        d["dst"][d["dst_space"] == 0] += np.uint64(base)
        s = torch.cuda.current_stream(self.dev).cuda_stream if stream is None else stream
        ft.submit_static(self.pool, d, weights, int(chunk_bytes), int(flags), s)

    def merge(self, open_job, descs, weights, flags=0, stream=None):
        d = np.array(descs, copy=True)
        base = self.host.data_ptr() if self.host is not None else 0
        d["src"][d["src_space"] == 0] += np.uint64(base)
        d["dst"][d["dst_space"] == 0] += np.uint64(base)
        if np.any(d["src_space"] == 2):
            d["src"][d["src_space"] == 2] += np.uint64(self.pageable_np.ctypes.data)
        if np.any(d["dst_space"] == 2):
            d["dst"][d["dst_space"] == 2] += np.uint64(self.pageable_np.ctypes.data)
        s = torch.cuda.current_stream(self.dev).cuda_stream if stream is None else stream
        return ft.submit_merge(self.pool, open_job, d, weights, int(flags), s)

    def wait(self, job):
        ft.wait(self.pool, job)

    def job_schedule(self, job, cls):
        return ft.job_schedule(self.pool, job, cls)

    def close_pool(self):
        """Destroy the pool handle; with reuse_memory the memory stays for the next pool."""
        if self.pool is not None:
            ft.pool_destroy(self.pool)
            self.pool = None
        self.segments = []
        self._seg_next = 0

    def close(self):
        if self.pool is not None:
            torch.cuda.synchronize(self.dev)
        self.close_pool()
        self._seg_cache = []
        self.host = None
        self.host_np = None
