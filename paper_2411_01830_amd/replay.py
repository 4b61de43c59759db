"""A workload replayed through the C ABI: what bench.py times and what the timeline tool looks at."""
import time

import numpy as np

class Replay:
    """A workload made concrete once (memory allocated and filled, descriptors resolved
    to addresses), then replayed step after step through the C ABI alone."""

    def __init__(self, name, detached):
        import torch
        from paper_2411_01830_amd import binding as ft, harness
        from workloads import configs, runner
        self.ft = ft
        self.torch = torch
        self.name = name
        self.plan = configs.CONFIGS[name](1.0)
        self.eng = harness.GpuEngine(0, reuse_memory=True)
        rec = runner.run_plan(self.plan, self.eng, flags=ft.FT_VALIDATE)     # fills inputs, checks aliasing once
        torch.cuda.synchronize()
        self.rec = rec
        self.segs = list(self.eng._seg_cache)
        self.host = self.eng.host
        self.eng.close_pool()
        base = np.uint64(self.host.data_ptr())
        self.ops = []
        for st in self.plan.steps:
            if st[0] == "alloc":
                self.ops.append(("alloc", int(st[2]), rec.alloc_off[st[1]]))
            elif st[0] == "submit":
                d = rec.descs[st[1]].copy()
                d["src"][d["src_space"] == 0] += base
                d["dst"][d["dst_space"] == 0] += base
                self.ops.append(("submit", st[1], d, np.asarray(st[3], dtype=np.uint32), int(st[4])))
            elif st[0] == "wait":
                self.ops.append(("wait", st[1]))
        self.detached = detached
        self.payload = self.plan.payload_bytes()
        self.stream = torch.cuda.current_stream().cuda_stream

    def step(self, flags=0, collect=None, tuning=None, epoch=False):
        ft = self.ft
        pool = ft.pool_create(self.segs[0].data_ptr(), self.segs[0].numel(), self.plan.slab_bytes, 0)
        ft.host_window_add(pool, self.host.data_ptr(), self.host.numel())
        if epoch:
            ft.timing_epoch(pool, self.stream)      # the jobs' begin / end times count from here
        if tuning:
            for cls, (wg, tile) in tuning.items():
                ft.set_tuning(pool, cls, wg, tile)
        nseg = 1
        jobs = {}
        flags |= ft.FT_TIMING | (ft.FT_DETACHED if self.detached else 0)
        alloc_s = 0.0
        for op in self.ops:
            if op[0] == "alloc":
                t0 = time.perf_counter()
                while True:
                    try:
                        off = ft.slab_alloc(pool, op[1])
                        break
                    except ft.FtError as e:
                        if e.code != -2 or nseg >= len(self.segs):
                            raise
                        ft.pool_grow(pool, self.segs[nseg].data_ptr(), self.segs[nseg].numel())
                        nseg += 1
                alloc_s += time.perf_counter() - t0
                if off != op[2]:
                    raise RuntimeError("allocator is not deterministic")
            elif op[0] == "submit":
                jobs[op[1]] = ft.submit_transfers(pool, op[2], op[3], op[4], flags, self.stream)
            else:
                ft.wait(pool, jobs[op[1]])
        out = {}
        for name, job in jobs.items():
            out[name] = ft.job_stats(pool, job)
            if collect is not None:
                collect(name, pool, job, out[name])
            ft.job_release(pool, job)
        ft.pool_destroy(pool)
        return out, alloc_s

    def close(self):
        self.eng.close()
