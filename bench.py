#!/usr/bin/env python3
"""Benchmark of the transfer engine on one MI355X.

A step is one pass of the whole hot path over one synthetic workload: create the
pool over resident device memory, slab-allocate every buffer (growing the pool when
it runs full), validate/plan/submit every batch of transfers and wait for all of
them. Inputs (pinned host sources, pool-resident sources) are in place before the
timed region. The default workload is the large mixed one (1024 transfers, 8 GiB,
60 % host->pool and 40 % pool->pool, pool growing 1 -> 16 GiB in 16 waves); the other
four workloads are run once each for the ``per_workload`` block of the same line.

Prints ONE JSON line. ``value`` is payload bytes per second over the timed steps.
``roofline`` is for the pool->pool copy kernel (HBM bound): algorithmic bytes are
2 x payload (one read, one write), durations come from HIP timing events that the
library binds to every launch of the timed steps on the kernel's own stream (they read
the start and the end of that dispatch).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

from paper_2411_01830_amd.replay import Replay

METRIC = "aggregate GB/s (host->pool, pool->pool) as % of roofline; weighted-share error"
HBM_PEAK_GBS = 8000.0
# HBM bytes the profiler counted per algorithmic byte for the pool->pool kernel, per workload: two counter runs
# of this very command under rocprofv3 (FETCH_SIZE, then WRITE_SIZE, each scaled by a plain copy of known size),
# whose summaries are the files named here. Counters cannot be read from inside the run that is being timed, so
# the line carries these constants and says where they come from (`traffic_source`); tests/test_host_logic.py
# holds every constant against the figure in its file. Workloads without such a run report null.
TRAFFIC_PER_ALGO_BYTE = {
    "large_mixed": (1.0077, "profiles/pmc_hbm_traffic_pool_to_pool_large_mixed.md"),
    "feature": (1.0010, "profiles/pmc_hbm_traffic_pool_to_pool_feature.md"),
    "traffic_crops": (1.3749, "profiles/pmc_hbm_traffic_pool_to_pool_traffic_crops.md"),
}
EXTRA_BLOCKS = ("share_error_pool_to_pool", "share_error_pool_to_host", "batched_triggering", "pinned_ring",
                "single_transfers", "elastic_store", "path_planner")


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="large_mixed",
                    choices=["tiny", "traffic", "feature", "contended", "large_mixed"])
    ap.add_argument("--no-extras", action="store_true", help="skip the other workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--blocks", default=None,
                    help="comma-separated: run only these of the blocks that widen the path (" + ", ".join(EXTRA_BLOCKS) +
                         ") and none of the other workloads; for profiling one block")
    ap.add_argument("--path", default="kernel", choices=["kernel", "dma"])
    return ap.parse_args()


def busy_ms(intervals):
    """Length of the union of [begin, end] intervals (ms): the time in which at least one of the launches ran."""
    total, cur_b, cur_e = 0.0, None, None
    for b, e in sorted(intervals):
        if cur_e is None or b > cur_e:
            if cur_e is not None:
                total += cur_e - cur_b
            cur_b, cur_e = b, e
        else:
            cur_e = max(cur_e, e)
    if cur_e is not None:
        total += cur_e - cur_b
    return total


def time_steps(rp, steps, warmup, flags=0):
    """cls_ms: per link class the sum of the launches' own durations (events bound to each dispatch).
    cls_busy_ms: the time in which at least one launch of the class was running - the union of the launches'
    [begin, end] intervals on the device's clock. The two agree unless launches overlap, which those of
    detached jobs do (two streams per class)."""
    torch = rp.torch
    for _ in range(warmup):
        rp.step(flags, epoch=rp.detached)
    torch.cuda.synchronize()
    cls_ms = [0.0, 0.0, 0.0]
    cls_busy = [0.0, 0.0, 0.0]
    cls_bytes = [0, 0, 0]
    cls_launches = [0, 0, 0]
    submit_us = 0.0
    alloc_s = 0.0
    t0 = time.perf_counter()
    for _ in range(steps):
        stats, a = rp.step(flags, epoch=rp.detached)
        alloc_s += a
        spans = [[], [], []]
        for st in stats.values():
            submit_us += st.host_submit_us
            for c in range(3):
                if st.cls[c].payload_bytes:
                    cls_ms[c] += st.cls[c].device_ms
                    cls_bytes[c] += st.cls[c].payload_bytes
                    cls_launches[c] += 1
                    if st.cls[c].end_ms > 0:
                        spans[c].append((st.cls[c].begin_ms, st.cls[c].end_ms))
                    else:
                        spans[c].append((-1e9 - len(spans[c]) * 1e6, -1e9 - len(spans[c]) * 1e6 + st.cls[c].device_ms))
        for c in range(3):
            cls_busy[c] += busy_ms(spans[c])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return {"wall_s": wall, "cls_ms": cls_ms, "cls_busy_ms": cls_busy, "cls_bytes": cls_bytes, "cls_launches": cls_launches,
            "submit_us_per_step": submit_us / steps, "alloc_us_per_step": alloc_s * 1e6 / steps}


def link_peak():
    """Best large pinned hipMemcpyAsync in each direction, measured now (GB/s)."""
    import torch
    n = 1 << 30
    h = torch.empty(n, dtype=torch.uint8, pin_memory=True)
    d = torch.empty(n, dtype=torch.uint8, device="cuda:0")
    out = {}
    for key, fn in (("h2d", lambda: d.copy_(h, non_blocking=True)), ("d2h", lambda: h.copy_(d, non_blocking=True))):
        best = 0.0
        fn()
        torch.cuda.synchronize()
        for _ in range(5):
            s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            s.record()
            fn()
            e.record()
            torch.cuda.synchronize()
            best = max(best, n / s.elapsed_time(e) / 1e6)
        out[key] = best
    return out


def plain_copy_ceiling():
    """Plain grid-stride kernels on 2 GiB, one workgroup per CU: a copy, reads alone and writes alone (GB/s of
    traffic). With read rate R and write rate W a copy cannot beat 2 / (1/R + 1/W)."""
    import torch
    from paper_2411_01830_amd import binding as ft
    n = 2 << 30
    a = torch.empty(n, dtype=torch.uint8, device="cuda:0")
    b = torch.empty(n, dtype=torch.uint8, device="cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    legs = {"copy": (lambda: ft.plain_copy(b.data_ptr(), a.data_ptr(), n, 256, st), 2 * n),
            "read": (lambda: ft.plain_read(a.data_ptr(), n, 256, st), n),
            "write": (lambda: ft.plain_fill(b.data_ptr(), n, 0x5A5A5A5A, 256, st), n)}
    best = {k: 0.0 for k in legs}
    for _ in range(6):
        for k, (fn, traffic) in legs.items():
            s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            s.record()
            fn()
            e.record()
            torch.cuda.synchronize()
            best[k] = max(best[k], traffic / s.elapsed_time(e) / 1e6)
    best["copy_bound"] = 2.0 / (1.0 / best["read"] + 1.0 / best["write"])
    return best


def share_error(rp, cls):
    """Timed per-function shares of one link class from the device log of one step:
    over [0, T1], T1 = first time any function's last byte lands."""
    ft = rp.ft
    got = {}

    def collect(name, pool, job, st):
        got["log"] = ft.job_log(pool, job, cls)
        got["weights"] = rp.rec.weights[name]

    rp.step(ft.FT_LOG, collect)
    return shares_from_log(got["log"], got["weights"], 512 << 10)


def _share_errors(t_begin0, t_end, func, nbytes, w):
    """max over active functions of |share - weight share| / weight share, over [0, T1] and per tenth of it;
    T1 = first time any function's last byte lands. Returns (T1 - t0, error, per-tenth errors, tickets in window)."""
    F = len(w)
    last = np.array([t_end[func == f].max() if np.any(func == f) else np.iinfo(np.int64).max for f in range(F)])
    T1 = int(last.min())
    active = np.array([np.any(func == f) for f in range(F)])
    want = w * active / (w * active).sum()

    def err_at(lo, hi):
        m = (t_end > lo) & (t_end <= hi)
        b = np.array([nbytes[m & (func == f)].sum() for f in range(F)], dtype=np.float64)
        if b.sum() == 0:
            return None
        share = b / b.sum()
        return float(np.max(np.abs(share - want)[active] / want[active]))

    t0 = t_begin0
    tenths = [err_at(t0 + (T1 - t0) * i // 10, t0 + (T1 - t0) * (i + 1) // 10) for i in range(10)]
    return T1 - t0, err_at(t0 - 1, T1), tenths, int(np.sum(t_end <= T1))


def shares_from_log(log, weights, chunk_bytes=None):
    """Timed shares from the copy kernel's own record (times, and the function each ticket was decoded to, both
    written by the kernel). Beside every timed figure the same statistic for the ticket order alone: the tickets
    in the order the device decoded them, completing one after the other at a uniform byte rate - what the chunk
    grain of the order contributes to the error before any timing effect."""
    w = np.asarray(weights, dtype=np.float64)
    func = log["func"].astype(np.int64)
    nbytes = log["bytes"].astype(np.int64)
    t_end = log["t_end_ns"].astype(np.int64)
    span, err, tenths, ntick = _share_errors(int(log["t_begin_ns"].min()), t_end, func, nbytes, w)
    ideal_end = np.cumsum(nbytes)
    _, err_o, tenths_o, _ = _share_errors(0, ideal_end, func, nbytes, w)
    rnd = lambda xs: [None if x is None else round(x, 4) for x in xs]
    return {"window": "[0,T1], T1 = first function done", "T1_ms": span / 1e6, "tickets_in_window": ntick,
            "max_rel_err": err, "max_rel_err_tenths": rnd(tenths),
            "order_alone": {"what": "same tickets in the decoded order at a uniform byte rate",
                            "max_rel_err": err_o, "max_rel_err_tenths": rnd(tenths_o)},
            "weights": [int(x) for x in w],
            **({"fluid_lag": lag_from_log(log, weights, chunk_bytes)} if chunk_bytes else {})}


def fluid_lag(func, nbytes, w, chunk_bytes, order):
    """How far every function is from its exact weighted share while the tickets complete in `order`: after each
    completion, bytes_f done so far against the fluid allocation of the total done so far - a_f = min(S_f, w_f * x)
    with x such that the a_f add up to the total (a function that has run dry leaves its part to the others in
    proportion). Unlike a share over one window this is defined at every instant and for any mix of stream sizes.
    Returns (largest |bytes_f - a_f| in chunks, its 99th percentile over completions and functions)."""
    w = np.asarray(w, dtype=np.float64)
    F = len(w)
    S = np.array([nbytes[func == f].sum() for f in range(F)], dtype=np.float64)
    act = S > 0
    if not act.any():
        return None, None
    lam = np.where(act, S / w, 0.0)
    by = np.argsort(lam)
    by = by[act[by]]
    lam_s, w_s, S_s = lam[by], w[by], S[by]
    # total bytes handed out when x reaches the i-th breakpoint; weight still active before it
    W_before = np.concatenate(([w_s.sum()], w_s.sum() - np.cumsum(w_s)[:-1]))
    B_at = np.array([np.minimum(S_s, w_s * l).sum() for l in lam_s])
    lam_prev = np.concatenate(([0.0], lam_s[:-1]))
    B_prev = np.concatenate(([0.0], B_at[:-1]))
    fo, bo = func[order], nbytes[order].astype(np.float64)
    total = np.cumsum(bo)
    seg = np.minimum(np.searchsorted(B_at, total, side="left"), len(B_at) - 1)
    x = lam_prev[seg] + (total - B_prev[seg]) / W_before[seg]
    done = np.zeros((len(fo), F))
    done[np.arange(len(fo)), fo] = bo
    done = np.cumsum(done, axis=0)
    fluid = np.minimum(S[None, :], w[None, :] * x[:, None])
    lag = np.abs(done - fluid)[:, act] / float(chunk_bytes)
    return float(lag.max()), float(np.percentile(lag, 99))


def lag_from_log(log, weights, chunk_bytes):
    """fluid_lag of the tickets in the order they completed on the device clock, and in the order they were decoded
    (ticket order: what the chunk order alone gives; anything beyond it is tiles in flight completing out of turn)."""
    func, nbytes = log["func"].astype(np.int64), log["bytes"].astype(np.int64)
    timed = fluid_lag(func, nbytes, weights, chunk_bytes, np.argsort(log["t_end_ns"], kind="stable"))
    alone = fluid_lag(func, nbytes, weights, chunk_bytes, np.arange(len(func)))
    r = lambda v: None if v is None else round(v, 3)
    return {"unit": "chunks", "timed_max": r(timed[0]), "timed_p99": r(timed[1]),
            "order_alone_max": r(alone[0]), "order_alone_p99": r(alone[1])}


def share_error_large_mixed(rp):
    """Timed shares where both kernels run side by side: one step of large_mixed with the per-ticket record, every
    wave's host->pool and pool->pool launch on its own. A wave holds some 38 + 26 transfers of 16 functions with
    lognormal sizes from 4 KiB up, so the first function is done after a handful of tickets and a share over
    [0, T1] says nothing here; reported instead, per class, is the distance of every function from its fluid
    weighted share at every completion (fluid_lag), the worst wave and the median wave."""
    ft = rp.ft
    per = {0: [], 2: []}

    def collect(name, pool, job, st):
        for cls in per:
            if st.cls[cls].payload_bytes:
                per[cls].append((ft.job_log(pool, job, cls), rp.rec.weights[name], st.cls[cls].tile_bytes * st.cls[cls].workgroups))

    rp.step(ft.FT_LOG, collect)
    chunk = 2 << 20
    out = {"what": "one step, FT_LOG; per wave and class the largest distance (in 2 MiB chunks) of any function from "
                   "its fluid weighted share at any completion; order_alone = the same tickets completing in ticket order",
           "chunk_bytes": chunk}
    for cls, name in ((0, "h2p"), (2, "p2p")):
        lags = [lag_from_log(log, weights, chunk) for log, weights, _ in per[cls]]
        in_flight = per[cls][0][2] if per[cls] else 0       # one tile per workgroup
        out[name] = {"waves": len(lags),
                     "timed_max_chunks": {"median_wave": round(float(np.median([l["timed_max"] for l in lags])), 3),
                                          "worst_wave": max(l["timed_max"] for l in lags)},
                     "timed_p99_chunks_median_wave": round(float(np.median([l["timed_p99"] for l in lags])), 3),
                     "order_alone_max_chunks": {"median_wave": round(float(np.median([l["order_alone_max"] for l in lags])), 3),
                                                "worst_wave": max(l["order_alone_max"] for l in lags)},
                     "in_flight_chunks": round(in_flight / chunk, 3)}
    return out


def share_error_pool_to_host():
    """The same measure on the link's other direction: 16 functions (weights from {1,2,4}, seeded) each send 64 MiB
    from the pool to pinned host memory in 512 KiB chunks, one job."""
    import torch
    from paper_2411_01830_amd import binding as ft
    from workloads import make_descs, FT_HOST, FT_POOL
    nf, per, chunk = 16, 64 << 20, 512 << 10
    rng = np.random.Generator(np.random.PCG64(241101830 + 11))
    w = [int(x) for x in rng.choice([1, 2, 4], nf)]
    buf = torch.empty(nf * per, dtype=torch.uint8, device="cuda:0")
    host = torch.empty(nf * per, dtype=torch.uint8, pin_memory=True)
    pool = ft.pool_create(buf.data_ptr(), buf.numel(), 1 << 20, 0)
    ft.host_window_add(pool, host.data_ptr(), host.numel())
    src = [ft.slab_alloc(pool, per) for _ in range(nf)]
    d = make_descs([dict(func=f, src_space=FT_POOL, dst_space=FT_HOST, src=src[f], dst=host.data_ptr() + f * per, row_bytes=per)
                    for f in range(nf)])
    stream = torch.cuda.current_stream().cuda_stream
    ft.wait(pool, ft.submit_transfers(pool, d, w, chunk, 0, stream))      # the device's first writes into the fresh arena
    job = ft.submit_transfers(pool, d, w, chunk, ft.FT_LOG | ft.FT_TIMING, stream)
    ft.wait(pool, job)
    out = shares_from_log(ft.job_log(pool, job, 1), w, chunk)
    out["payload_GBps"] = round(nf * per / ft.job_stats(pool, job).cls[1].device_ms / 1e6, 2)
    ft.job_release(pool, job)
    ft.pool_destroy(pool)
    return out


def share_error_pool_to_pool():
    """The same measure for the on-device class: eight functions with the feature workload's weights
    (1:1:2:2:4:4:8:8), each moving 1 GiB between slabs in 2 MiB chunks, so that the window in which all
    eight are active holds some two thousand chunks (in the feature workload itself it is 29 us long and
    a weight-1 function moves one or two chunks in it)."""
    import torch
    from paper_2411_01830_amd import binding as ft
    from workloads import make_descs, FT_POOL
    nf, per = 8, 1 << 30
    w = [1, 1, 2, 2, 4, 4, 8, 8]
    buf = torch.empty(2 * nf * per, dtype=torch.uint8, device="cuda:0")
    pool = ft.pool_create(buf.data_ptr(), buf.numel(), 1 << 20, 0)
    src = [ft.slab_alloc(pool, per) for _ in range(nf)]
    dst = [ft.slab_alloc(pool, per) for _ in range(nf)]
    d = make_descs([dict(func=f, src_space=FT_POOL, dst_space=FT_POOL, src=src[f], dst=dst[f], row_bytes=per)
                    for f in range(nf)])
    stream = torch.cuda.current_stream().cuda_stream
    ft.wait(pool, ft.submit_transfers(pool, d, w, 2 << 20, 0, stream))      # touch everything once
    job = ft.submit_transfers(pool, d, w, 2 << 20, ft.FT_LOG | ft.FT_TIMING, stream)
    ft.wait(pool, job)
    out = shares_from_log(ft.job_log(pool, job, 2), w, 2 << 20)
    gbps = nf * per / ft.job_stats(pool, job).cls[2].device_ms / 1e6
    out["payload_GBps"] = round(gbps, 1)
    out["hbm_frac"] = round(2 * gbps / HBM_PEAK_GBS, 4)      # with the per-ticket log being written
    ft.job_release(pool, job)
    ft.pool_destroy(pool)
    return out


def batched_triggering(peaks):
    """Sec. 6.1 on the contended host link: 16 background functions stream 256 MiB each
    (objective 1 s, 0.1 s of it inference); 10 ms into the job an urgent function arrives
    with 8 MiB, a 3 ms objective and 1 ms of inference. Weights come from the rate-control
    rule (ft_slo_weights, link = the measured peak). Closed job: the newcomer queues behind
    the 4 GiB. Open job: it joins at the next batch. Reports the newcomer's transfer latency
    (merge call to wait) and what batching costs the background job."""
    import torch
    from paper_2411_01830_amd import binding as ft
    from workloads import make_descs
    rp = Replay("contended", False)
    sub = [o for o in rp.ops if o[0] == "submit"][0]
    descs, chunk = sub[2], sub[4]
    allocs = [o for o in rp.ops if o[0] == "alloc"]
    nbg, small = len(sub[3]), 8 << 20
    sizes = [float(256 << 20)] * nbg + [float(small)]
    rates, w = ft.slo_weights(sizes, [1.0] * nbg + [0.003], [0.1] * nbg + [0.001], peaks["h2d"] * 1e9)
    out = {"weights_background": w[0], "weight_urgent": w[-1], "urgent_rate_GBps": round(rates[-1] / 1e9, 2),
           "urgent_budget_ms": 2.0, "urgent_bytes": small, "chunk_bytes": chunk, "cases": {}}
    for name, batch in (("closed", 0), ("open_batch5", 5), ("open_batch20", 20)):
        lat, tot = [], []
        for _ in range(3):
            pool = ft.pool_create(rp.segs[0].data_ptr(), rp.segs[0].numel(), rp.plan.slab_bytes, 0)
            ft.host_window_add(pool, rp.host.data_ptr(), rp.host.numel())
            for a in allocs:
                ft.slab_alloc(pool, a[1])
            off = ft.slab_alloc(pool, small)
            urgent = make_descs([dict(func=0, src_space=0, dst_space=1, src=rp.host.data_ptr() + 4096, dst=off,
                                      row_bytes=small)])
            if batch:
                ft.set_batch(pool, batch, 3)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            j1 = ft.submit_transfers(pool, descs, w[:nbg], chunk, ft.FT_OPEN if batch else ft.FT_DETACHED, rp.stream)
            time.sleep(0.010)
            t1 = time.perf_counter()
            if batch:
                j2 = ft.submit_merge(pool, j1, urgent, w[-1:], 0, rp.stream)
            else:
                j2 = ft.submit_transfers(pool, urgent, w[-1:], chunk, ft.FT_DETACHED, rp.stream)
            ft.wait(pool, j2)
            t2 = time.perf_counter()
            ft.wait(pool, j1)
            t3 = time.perf_counter()
            lat.append((t2 - t1) * 1e3)
            tot.append((t3 - t0) * 1e3)
            ft.pool_destroy(pool)
        lat.sort()
        tot.sort()
        out["cases"][name] = {"urgent_latency_ms": round(lat[1], 3), "background_ms": round(tot[1], 2),
                              "background_GBps": round(rp.payload / tot[1] / 1e6, 2),
                              "urgent_within_budget": bool(lat[1] <= 2.0)}
    # rate control on the running sequence: all 16 equal, 10 ms in function 0 gets 8 of 23 parts
    pool = ft.pool_create(rp.segs[0].data_ptr(), rp.segs[0].numel(), rp.plan.slab_bytes, 0)
    ft.host_window_add(pool, rp.host.data_ptr(), rp.host.numel())
    for a in allocs:
        ft.slab_alloc(pool, a[1])
    ft.set_batch(pool, 5, 3)
    torch.cuda.synchronize()
    job = ft.submit_transfers(pool, descs, [1] * nbg, chunk, ft.FT_OPEN | ft.FT_KEEP, rp.stream)
    time.sleep(0.010)
    t0 = time.perf_counter()
    at = ft.job_reweight(pool, job, [8] + [1] * (nbg - 1), rp.stream)[0]
    call_us = (time.perf_counter() - t0) * 1e6
    ft.wait(pool, job)
    batches = ft.job_batches(pool, job, 0)
    if at is not None:
        before = [f for b in batches[:at] for _, f, _ in b]
        last0 = max(i for i, b in enumerate(batches) if any(f == 0 for _, f, _ in b))
        after = [f for b in batches[at:last0] for _, f, _ in b]
        out["reweight"] = {"call_us": round(call_us, 1), "from_batch": at, "batches": len(batches),
                           "share_before": round(before.count(0) / max(len(before), 1), 4), "want_before": round(1 / nbg, 4),
                           "share_after": round(after.count(0) / max(len(after), 1), 4),
                           "want_after": round(8 / (8 + nbg - 1), 4), "function0_done_at_batch": last0}
    ft.job_release(pool, job)
    ft.pool_destroy(pool)
    rp.close()
    return out


def reserve_rings():
    """The pinned rings of the `pinned_ring` leg, taken at the start of the process as a long-running server
    would (ft_reserve_rings; the library keeps a ring's memory for the life of the process). Pinned memory that
    the runtime hands out after other large pinned allocations have come and gone takes device writes at
    46 GB/s here, memory taken early at 53-54."""
    import torch
    from paper_2411_01830_amd import binding as ft
    seg = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
    pool = ft.pool_create(seg.data_ptr(), seg.numel(), 1 << 20, 0)
    ft.set_batch(pool, 5, 3)
    ft.reserve_rings(pool, 2 << 20)
    ft.pool_destroy(pool)


def pinned_ring(peaks):
    """Sec. 6.1, circular pinned buffer: 1 GiB of four functions from ordinary (pageable) host
    memory into the pool through the open job's ring (2 MiB chunks, batches of 5, 3 queued
    ahead: a 40 MiB ring), against the runtime's own copy from pageable memory."""
    import torch
    from paper_2411_01830_amd import binding as ft, harness
    from workloads import make_descs
    total, nf, chunk = 1 << 30, 4, 2 << 20
    eng = harness.GpuEngine()
    eng.host_arena(4096)
    eng.pageable_arena(total, fill=7)
    eng.pool_create(total + (64 << 20), 1 << 20, fill=None)
    per = total // nf
    d = make_descs([dict(func=f, src_space=2, dst_space=1, src=f * per, dst=eng.slab_alloc(per), row_bytes=per)
                    for f in range(nf)])
    out = {"bytes": total, "chunk_bytes": chunk, "batch_chunks": 5, "depth": 3, "ring_MiB": 40,
           "ring_memory": "taken at the start of the process (ft_reserve_rings)", "ring_GBps": {}}
    for threads in (1, 4, 8):
        ft.set_batch(eng.pool, 5, 3)
        ft.set_stage_threads(eng.pool, threads)
        ts = []
        for _ in range(3):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            eng.wait(eng.submit(d, [1] * nf, chunk, ft.FT_OPEN))
            ts.append(time.perf_counter() - t0)
        ts.sort()
        out["ring_GBps"][f"{threads}_threads"] = round(total / ts[1] / 1e9, 2)
    out["ring_4_threads_link_frac"] = round(out["ring_GBps"]["4_threads"] / peaks["h2d"], 4)
    # the other direction: pool -> ordinary host memory
    back = make_descs([dict(func=f, src_space=1, dst_space=2, src=int(d["dst"][f]), dst=f * per, row_bytes=per)
                       for f in range(nf)])
    ft.set_stage_threads(eng.pool, 4)
    ts = []
    for _ in range(3):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        eng.wait(eng.submit(back, [1] * nf, chunk, ft.FT_OPEN))
        ts.append(time.perf_counter() - t0)
    ts.sort()
    out["to_pageable"] = {"ring_4_threads_GBps": round(total / ts[1] / 1e9, 2),
                          "ring_link_frac": round(total / ts[1] / 1e9 / peaks["d2h"], 4)}
    # the runtime's own copies between the same pageable memory and the device, measured last
    host_t = torch.from_numpy(eng.pageable_np)
    dev_t = torch.empty(total, dtype=torch.uint8, device="cuda:0")
    for key, dst, src in (("runtime_copy_from_pageable_GBps", dev_t, host_t), ("runtime_copy_to_pageable_GBps", host_t, dev_t)):
        best = 0.0
        for _ in range(3):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            dst.copy_(src)
            torch.cuda.synchronize()
            best = max(best, total / (time.perf_counter() - t0) / 1e9)
        out[key] = round(best, 2)
    del dev_t
    eng.close()
    return out


def single_transfers():
    """Wall time from submit to the end of wait for one contiguous transfer, per link class and
    size, against the runtime's own copy (`Tensor.copy_` + stream synchronize) of the same bytes:
    what passing one tensor costs (Sec. 2.2 measures passing latency, not only bandwidth)."""
    import torch
    from paper_2411_01830_amd import binding as ft
    from workloads import make_descs, FT_HOST, FT_POOL
    cap = 64 << 20
    host = torch.empty(cap, dtype=torch.uint8, pin_memory=True)
    buf = torch.empty(2 * cap, dtype=torch.uint8, device="cuda:0")
    pool = ft.pool_create(buf.data_ptr(), 2 * cap, 1 << 20, 0)
    ft.host_window_add(pool, host.data_ptr(), cap)
    a, b = ft.slab_alloc(pool, cap), ft.slab_alloc(pool, cap)
    stream = torch.cuda.current_stream().cuda_stream

    def med(f, n=25):
        ts = []
        for _ in range(n + 3):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            f()
            ts.append(time.perf_counter() - t0)
        ts = sorted(ts[3:])
        return round(ts[len(ts) // 2] * 1e6, 1)
    out = {"unit": "us, median of 25, submit -> wait returns", "sizes": {}}
    hp = host.data_ptr()
    import numpy as np
    page = np.zeros(8 << 20, dtype=np.uint8)          # ordinary host memory
    ft.pageable_window_add(pool, page.ctypes.data, len(page))
    page_t = torch.from_numpy(page)
    for n in (64 << 10, 1 << 20, 16 << 20, 64 << 20):
        row = {}
        if n <= len(page):
            # from pageable memory without an open job: through the job's own pinned buffer
            dp = ft.Transfers(make_descs([dict(func=0, src_space=2, dst_space=FT_POOL, src=page.ctypes.data, dst=a,
                                                 row_bytes=n)]), [1])
            bn, pn = buf[:n], page_t[:n]

            def engine_pageable():
                ft.wait(pool, ft.submit_transfers(pool, dp, None, 2 << 20, 0, stream))

            def runtime_pageable():
                bn.copy_(pn)
                torch.cuda.current_stream().synchronize()
            row["pageable_to_pool"] = {"engine": med(engine_pageable), "runtime_copy": med(runtime_pageable)}
        for name, ss, ds, src, dst, tsrc, tdst in (("host_to_pool", FT_HOST, FT_POOL, hp, a, host, buf),
                                                   ("pool_to_host", FT_POOL, FT_HOST, a, hp, buf, host),
                                                   ("pool_to_pool", FT_POOL, FT_POOL, a, b, buf, buf[cap:])):
            # both sides prepared outside the timed call: descriptors marshalled once, tensor views sliced once
            d = ft.Transfers(make_descs([dict(func=0, src_space=ss, dst_space=ds, src=src, dst=dst, row_bytes=n)]), [1])
            dn, sn = tdst[:n], tsrc[:n]

            def engine():
                ft.wait(pool, ft.submit_transfers(pool, d, None, 2 << 20, 0, stream))

            def runtime():
                dn.copy_(sn, non_blocking=True)
                torch.cuda.current_stream().synchronize()
            row[name] = {"engine": med(engine), "runtime_copy": med(runtime)}
        out["sizes"][f"{n >> 10}_KiB"] = row
    ft.pool_destroy(pool)
    return out


def elastic_store():
    """Sec. 7 with the library's host-side policies on synthetic traces (the paper's Azure trace
    is not available; seeded arrivals with quiet and bursty periods and lognormal result sizes
    stand in for it). Pool sizing: reserved bytes over time under the histogram rule against a
    caching pool that never gives memory back, and how often a result fitted into what was
    reserved when it arrived. Migration: consumers that found their input moved out to host
    memory, queue-aware against least-recently-stored eviction. Also the cost of the
    allocation calls themselves against native device allocation."""
    import torch
    from paper_2411_01830_amd import binding as ft
    from workloads import traces
    rng = np.random.Generator(np.random.PCG64(241101830 + 7))
    # ---- pool sizing
    sizer = ft.Sizer(300 << 20, 0.99, 60.0)
    horizon = 3600.0
    events = traces.sizing_trace(rng, horizon)
    reserved_sum = held_sum = peak = 0.0
    hits = 0
    last_t, cur, held = 0.0, sizer.target(0.0), 300 << 20
    for (t, f, size, con) in events:
        if t >= horizon:
            break
        cur = sizer.target(t)
        hits += size * con <= cur
        reserved_sum += cur * (t - last_t)
        held = max(held, cur)
        held_sum += held * (t - last_t)
        peak = max(peak, cur)
        last_t = t
        sizer.observe(f, t, size, con)
    sizer.close()
    sizing = {"trace": "3 functions, 3600 s; two are busy for 300 s in every 1200 s and nearly idle otherwise, one is steady; lognormal sizes (synthetic)",
              "requests": len(events), "mean_reserved_MiB": round(reserved_sum / last_t / 2**20, 1),
              "never_release_mean_MiB": round(held_sum / last_t / 2**20, 1), "peak_MiB": round(peak / 2**20, 1),
              "memory_vs_never_release": round(reserved_sum / held_sum, 3),
              "requests_fitting_reservation": round(hits / len(events), 3)}
    # ---- migration
    n, look, cap = 2000, 12, 1 << 30
    sizes = traces.result_sizes(rng, n, 96 << 20, 0.7, 1 << 20, 512 << 20)

    def simulate(policy):
        r = traces.two_stage_queue(sizes, cap, look, lambda objs, capacity, incoming: ft.migrate_plan(objs, capacity, incoming, policy))
        return r["stalls"], r["bytes_out"] + r["bytes_in"]
    qa, lru = simulate(ft.FT_EVICT_QUEUE_AWARE), simulate(ft.FT_EVICT_LRU)
    migration = {"trace": f"{n} requests of a two-stage workflow, producers {look} requests ahead, 1 GiB store, "
                          "lognormal results (median 96 MiB, synthetic)",
                 "queue_aware": {"stalled_consumers": qa[0], "GiB_moved": round(qa[1] / 2**30, 1)},
                 "least_recently_stored": {"stalled_consumers": lru[0], "GiB_moved": round(lru[1] / 2**30, 1)}}
    # ---- allocation cost
    seg = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
    pool = ft.pool_create(seg.data_ptr(), seg.numel(), 1 << 20, 0)
    t0 = time.perf_counter()
    offs = [ft.slab_alloc(pool, 8 << 20) for _ in range(100)]
    for o in offs:
        ft.slab_free(pool, o)
    pool_us = (time.perf_counter() - t0) / 200 * 1e6
    ft.pool_destroy(pool)
    del seg
    torch.cuda.empty_cache()
    t0 = time.perf_counter()
    for _ in range(10):
        x = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0")   # above every caching threshold
        del x
        torch.cuda.empty_cache()                                          # hands it back to the driver
    torch.cuda.synchronize()
    native_us = (time.perf_counter() - t0) / 10 * 1e6
    return {"pool_sizing": sizing, "migration": migration, "store_on_device": store_on_device(),
            "allocation": {"slab_alloc_or_free_us": round(pool_us, 2), "native_alloc_plus_free_256MiB_us": round(native_us, 1)}}


def store_on_device():
    """The library's store (ft_store_*) run on the GPU: a two-stage workflow whose producers run 24
    requests ahead of the consumers, lognormal results (median 48 MiB), 1 GiB of them allowed in the
    pool. What a request costs in store calls (moves included) and what the moves themselves reach."""
    import torch
    from paper_2411_01830_amd import binding as ft
    rng = np.random.Generator(np.random.PCG64(241101830 + 9))
    n, lookahead, cap = 150, 24, 1 << 30
    sizes = np.clip(np.exp(rng.normal(np.log(48 << 20), 0.8, n)), 1 << 20, 400 << 20).astype(np.int64) // 4096 * 4096
    pool_bytes, spill_bytes = 2 << 30, 4 << 30
    dev = torch.empty(pool_bytes, dtype=torch.uint8, device="cuda:0")
    host = torch.empty(spill_bytes, dtype=torch.uint8, pin_memory=True)
    # twice: the first pass also pays for the device's first writes into the fresh pinned arena
    # (moves out at 25 GB/s instead of 55)
    for _ in range(2):
        pool = ft.pool_create(dev.data_ptr(), pool_bytes, 1 << 20, 0)
        store = ft.Store(pool, host.data_ptr(), spill_bytes, cap, 2 << 20, torch.cuda.current_stream().cuda_stream)
        stored = 0
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for head in range(n):
            while stored < n and stored <= head + lookahead:
                store.put(stored, int(sizes[stored]), stored - head)
                stored += 1
            store.get(head)
            store.done(head)
            store.advance(1)
        calls = time.perf_counter() - t0        # what the store's calls held the host for
        store.sync()
        wall = time.perf_counter() - t0         # until the last move was in place
        st = store.stats()
        store.close()
        ft.pool_destroy(pool)
    out = {"requests": n, "capacity_GiB": 1.0, "stored_GiB": round(float(sizes.sum()) / 2**30, 2),
           "moved_out": st.moved_out, "moved_in": st.moved_in, "stalled_consumers": st.stalls,
           "GiB_moved": round((st.bytes_out + st.bytes_in) / 2**30, 2),
           "ms_per_request_in_store_calls": round(calls * 1e3 / n, 3), "ms_per_request": round(wall * 1e3 / n, 3),
           "what": "moves are jobs on the store's stream that put/done do not wait for; get waits for the one "
                   "result it returns (the consumer here asks right away, so it waits for the moves queued before it)",
           "moves_GBps": round((st.bytes_out + st.bytes_in) / wall / 1e9, 1)}
    return out


def path_planner():
    """Sec. 6.2, Alg. 1 as a host-side planner (one GPU here, so nothing is moved): bandwidth of the
    parallel paths it finds on two synthetic 8-GPU topologies and what a selection costs."""
    from paper_2411_01830_amd import binding as ft
    from workloads import traces
    cube, mesh = traces.hybrid_cube_mesh_24_48(), traces.full_mesh(8, 64)
    out = {}
    for name, topo, hops, (s, d) in (("hybrid_cube_mesh_24_48", cube, 0, (0, 3)), ("full_mesh_64", mesh, 3, (0, 5))):
        links = ft.Links(topo, hops)
        paths = links.select(1, s, d)
        links.release(1)
        links.select(1, s, d)          # the candidate lists are cached from here on
        links.release(1)
        t0 = time.perf_counter()
        reps = 200
        for i in range(reps):
            ft._lib.ft_links_select(links._h, 2 + i, s, d)
            ft._lib.ft_links_release(links._h, 2 + i)
        us = (time.perf_counter() - t0) / reps * 1e6
        links.close()
        bw = [b for _, b in paths]
        out[name] = {"pair": [s, d], "direct_GBps": topo[s][d], "paths": len(paths), "parallel_GBps": sum(bw),
                     "select_plus_release_us": round(us, 1),
                     "first_chunks_to_paths": ft.stripe_chunks(bw, 12)}
    return out


def cpu_baseline():
    """The CPU oracle, as it stands, on a bounded sample of the same workload: the first
    waves of large_mixed at full size, as many as keep the leg around 10-30 s."""
    from oracle import OracleEngine
    from workloads import configs, runner
    full = configs.large_mixed(1.0)
    for waves in (4, 16):
        plan = configs.first_submits(full, waves)
        eng = OracleEngine()
        t0 = time.perf_counter()
        rec = runner.run_plan(plan, eng, fill=False)
        dt = time.perf_counter() - t0
        if dt >= 4.0 or waves == 16:
            break
        del eng, rec
    out = {"value": plan.payload_bytes() / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
           "sample": f"first {waves} of the 16 waves of large_mixed at full size "
                     f"({plan.payload_bytes() / 2**30:.2f} GiB payload, allocation and pool growth included), "
                     f"{dt:.1f} s, {os.cpu_count()} logical CPUs present"}
    # the same bytes once more, one thread per function: each thread writes its function's descriptors
    # straight from the definition (the oracle's apply_definition; NumPy slice copies release the lock)
    import threading
    import numpy as np
    per_func = {}
    for d in rec.descs.values():
        for f in np.unique(d["func"]):
            per_func.setdefault(int(f), []).append(d[d["func"] == f])
    threads = [threading.Thread(target=lambda ds=ds: [eng.apply_definition(x) for x in ds]) for ds in per_func.values()]
    t0 = time.perf_counter()
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    dt2 = time.perf_counter() - t0
    out["parallel_variant"] = {"value": plan.payload_bytes() / dt2 / 1e9, "unit": "GB/s", "threads": len(threads),
                               "what": "byte movement only (every buffer in host memory, no link crossed), one thread per function, same sample"}
    return out


def sector_bytes(rp):
    """Pool->pool descriptors of pitched rows (the traffic workload's crops): the bytes of all 64-byte and
    128-byte lines that the rows touch on the read side and on the write side, beside the payload. Rows of
    64-256 bytes at any alignment touch up to one line more than their length fills."""
    out = {"payload": 0, "read_64": 0, "read_128": 0, "write_64": 0, "write_128": 0}
    for op in rp.ops:
        if op[0] != "submit":
            continue
        for d in op[2]:
            if d["src_space"] != 1 or d["dst_space"] != 1:
                continue
            rows, w = int(d["rows"]), int(d["row_bytes"])
            r = np.arange(rows, dtype=np.int64)
            out["payload"] += rows * w
            for side, base, pitch in (("read", int(d["src"]), int(d["src_pitch"])), ("write", int(d["dst"]), int(d["dst_pitch"]))):
                a = base + r * (pitch if rows > 1 else 0)
                for g in (64, 128):
                    lines = np.unique(np.concatenate([np.arange(x // g, (x + w - 1) // g + 1) for x in a])) \
                        if rows <= 4096 else None
                    out[f"{side}_{g}"] += int(len(lines)) * g if lines is not None else (w + g - 1) // g * g * rows
    return out


def summarize(name, res, steps, rp, peaks):
    ms_per_step = res["wall_s"] * 1e3 / steps
    out = {"payload_GiB": round(rp.payload / 2**30, 3), "ms_per_step": round(ms_per_step, 3),
           "GBps": round(rp.payload * steps / res["wall_s"] / 1e9, 2),
           "submit_us_per_step": round(res["submit_us_per_step"], 1),
           "alloc_us_per_step": round(res["alloc_us_per_step"], 1)}
    names = ("h2p", "p2h", "p2p")
    for c in range(3):
        if res["cls_bytes"][c] == 0:
            continue
        gbps = res["cls_bytes"][c] / res["cls_busy_ms"][c] / 1e6          # over the time the class was busy
        entry = {"payload_GBps": round(gbps, 2), "launches": res["cls_launches"][c],
                 "avg_launch_ms": round(res["cls_ms"][c] / res["cls_launches"][c], 4),
                 "busy_ms_per_launch": round(res["cls_busy_ms"][c] / res["cls_launches"][c], 4)}
        if c == 2:
            entry["hbm_frac"] = round(2 * gbps / HBM_PEAK_GBS, 4)
            entry["hbm_frac_per_dispatch"] = round(2 * res["cls_bytes"][c] / res["cls_ms"][c] / 1e6 / HBM_PEAK_GBS, 4)
            if name == "traffic":
                sb = sector_bytes(rp)
                entry["line_granular_bytes_per_payload_byte"] = {
                    "lines_64B": round((sb["read_64"] + sb["write_64"]) / (2 * sb["payload"]), 4),
                    "lines_128B": round((sb["read_128"] + sb["write_128"]) / (2 * sb["payload"]), 4),
                    "measured_hbm_traffic": TRAFFIC_PER_ALGO_BYTE["traffic_crops"][0],
                    "measured_hbm_traffic_source": TRAFFIC_PER_ALGO_BYTE["traffic_crops"][1] + " (counter runs of "
                                                   "`bench.py --workload traffic`, not this run)"}
                entry["hbm_frac_line_granular_128B"] = round(
                    gbps * (sb["read_128"] + sb["write_128"]) / sb["payload"] / HBM_PEAK_GBS, 4)
        else:
            entry["link_frac"] = round(gbps / peaks["h2d" if c == 0 else "d2h"], 4)
        out[names[c]] = entry
    return out


def main():
    args = parse_args()
    if args.blocks is not None:
        args.blocks = [b for b in args.blocks.split(",") if b]
        unknown = [b for b in args.blocks if b not in EXTRA_BLOCKS]
        if unknown:
            print(f"bench.py: unknown block(s) {unknown}; known: {', '.join(EXTRA_BLOCKS)}", file=sys.stderr)
            sys.exit(2)
        args.no_extras = True
    if args.gpus != 1:
        print("bench.py: this engine is a single-GPU build (one pool, one host link per GPU); "
              "run with --gpus 1. Several GPUs would run independent engines.", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU; there is no CPU path", file=sys.stderr)
        sys.exit(2)
    from paper_2411_01830_amd import binding as ft
    flags = ft.FT_PATH_DMA if args.path == "dma" else 0
    if not args.no_extras or (args.blocks and "pinned_ring" in args.blocks):
        reserve_rings()
    peaks = link_peak()
    ceiling = plain_copy_ceiling()

    detached = {"large_mixed": True}
    rp = Replay(args.workload, detached.get(args.workload, False))
    res = time_steps(rp, args.steps, args.warmup, flags)
    main_sum = summarize(args.workload, res, args.steps, rp, peaks)
    value = rp.payload * args.steps / res["wall_s"] / 1e9
    line = {
        "metric": METRIC, "value": round(value, 3), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(res["wall_s"] * 1e3 / args.steps, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8",
        "data": "synthetic",
        "config": {"workload": args.workload, "payload_bytes_per_step": rp.payload,
                   "path": args.path, "transfers": sum(len(o[2]) for o in rp.ops if o[0] == "submit"),
                   "submits_per_step": sum(1 for o in rp.ops if o[0] == "submit")},
    }
    # roofline of the pool->pool copy kernel; if this workload has none, of the feature workload below
    roof_src = res if res["cls_bytes"][2] else None
    roof_name = args.workload
    per = {args.workload: main_sum}
    shares = None
    dma = {}
    if not args.no_extras or roof_src is None:
        for other in ("feature", "contended", "traffic", "tiny"):
            if other == args.workload:
                if other == "contended":
                    shares = share_error(rp, 0)
                continue
            if args.no_extras and not (other == "feature" and roof_src is None):
                continue
            rq = Replay(other, False)
            k = 20 if other in ("feature", "tiny", "traffic") else 5
            r = time_steps(rq, k, 2, flags)
            per[other] = summarize(other, r, k, rq, peaks)
            if other == "feature" and roof_src is None:
                roof_src, roof_name = r, "feature"
            if args.path == "kernel" and other in ("contended", "feature"):
                # the same schedule through the copy engines, one runtime copy per chunk piece
                rd = time_steps(rq, 2, 1, ft.FT_PATH_DMA)
                dma[other] = {k2: v for k2, v in summarize(other, rd, 2, rq, peaks).items() if k2 in ("h2p", "p2h", "p2p")}
            if other == "contended":
                shares = share_error(rq, 0)
            rq.close()
    if roof_src is not None and roof_src["cls_bytes"][2]:
        algo = 2.0 * roof_src["cls_bytes"][2]
        traffic_factor, traffic_file = TRAFFIC_PER_ALGO_BYTE.get("traffic_crops" if roof_name == "traffic" else roof_name,
                                                                 (None, None))
        achieved = algo / roof_src["cls_busy_ms"][2] / 1e6
        per_dispatch = algo / roof_src["cls_ms"][2] / 1e6
        line["roofline"] = {
            "bound": "hbm", "kernel": "ft_copy_kernel<true, 2> (pool->pool)", "workload": roof_name,
            "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "time_base": "union of the launches' [begin, end] intervals on the device clock (launches of detached "
                         "jobs overlap on the class's two streams); per_dispatch_* divide by the sum of the "
                         "launches' own durations instead",
            "busy_ms_per_launch": round(roof_src["cls_busy_ms"][2] / roof_src["cls_launches"][2], 5),
            "per_dispatch_achieved": round(per_dispatch, 1), "per_dispatch_frac": round(per_dispatch / HBM_PEAK_GBS, 4),
            "algorithmic_bytes_per_launch": round(algo / roof_src["cls_launches"][2]),
            "avg_launch_ms": round(roof_src["cls_ms"][2] / roof_src["cls_launches"][2], 5),
            "launches": roof_src["cls_launches"][2],
            "traffic": None if traffic_factor is None else round(traffic_factor * algo / roof_src["cls_launches"][2]),
            "traffic_source": None if traffic_factor is None else
            f"{traffic_file}: {traffic_factor} HBM bytes per algorithmic byte, from rocprofv3 counter runs of this "
            "command (FETCH_SIZE, WRITE_SIZE, scaled by a plain copy of known size); not measured in this run",
            "plain_copy_ceiling_GBps": round(ceiling["copy"], 1),
            "plain_read_only_GBps": round(ceiling["read"], 1), "plain_write_only_GBps": round(ceiling["write"], 1),
            "copy_bound_from_those_GBps": round(ceiling["copy_bound"], 1),
            "frac_of_copy_bound": round(achieved / ceiling["copy_bound"], 4),
        }
    if res["cls_bytes"][0]:
        g = res["cls_bytes"][0] / res["cls_busy_ms"][0] / 1e6
        line["host_link"] = {"direction": "host->pool", "achieved": round(g, 2), "peak_measured": round(peaks["h2d"], 2),
                             "unit": "GB/s", "frac": round(g / peaks["h2d"], 4),
                             "peak_is": "best of 5 hipMemcpyAsync of 1 GiB pinned, same run",
                             "d2h_peak_measured": round(peaks["d2h"], 2)}
    if shares is not None:
        line["share_error"] = shares
    if args.workload == "large_mixed" and not args.no_extras:
        try:
            line["share_error_large_mixed"] = share_error_large_mixed(rp)
        except Exception as e:      # noqa: BLE001
            line["share_error_large_mixed"] = {"error": repr(e)}
    line["per_workload"] = per
    if dma:
        line["dma_path"] = {"what": "FT_PATH_DMA: same chunk order, one hipMemcpyAsync / hipMemcpy2DAsync per chunk piece "
                                    "(2 steps each); compare with per_workload", **dma}
    rp.close()
    if not args.no_extras or args.blocks:
        # the blocks that widen the path; one that fails must not take the headline figures with it
        blocks = {"share_error_pool_to_pool": share_error_pool_to_pool,
                  "share_error_pool_to_host": share_error_pool_to_host,
                  "batched_triggering": lambda: batched_triggering(peaks),
                  "pinned_ring": lambda: pinned_ring(peaks),
                  "single_transfers": single_transfers,
                  "elastic_store": elastic_store,
                  "path_planner": path_planner}
        for key in (args.blocks if args.blocks else EXTRA_BLOCKS):
            try:
                line[key] = blocks[key]()
            except Exception as e:      # noqa: BLE001
                line[key] = {"error": repr(e)}
                print(f"bench.py: block {key} failed: {e!r}", file=sys.stderr)
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
