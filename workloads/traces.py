"""Synthetic traces and topologies for the rows that widen the path (Sec. 6.2, Sec. 7): request arrivals with
result sizes, the two-stage workflow that puts a store under memory pressure, and two 8-GPU link graphs.

Inputs only. The policies they exercise (pool sizing, what to move out and back, which paths to take) are
passed in as callables or applied by the caller; nothing here decides anything. The paper's Azure trace and
its servers' link maps are not available: these stand in for them.
"""
import numpy as np


def sizing_trace(rng, horizon=3600.0):
    """Arrivals of three functions over `horizon` seconds: two are busy for 300 s in every 1200 s (4 and 1
    requests a second) and nearly idle otherwise, one is steady (one request every 2 s); result sizes are
    lognormal around 24, 96 and 6 MiB, clipped to [1 MiB, 1 GiB]; 1-4 results held at once in a burst, 1
    otherwise. Returns a time-sorted list of (t, function, bytes, concurrency)."""
    events = []
    for f, (rate_quiet, rate_burst, med) in enumerate(((0.002, 4.0, 24 << 20), (0.002, 1.0, 96 << 20),
                                                       (0.5, 0.5, 6 << 20))):
        t = 0.0
        while t < horizon:
            burst = (t // 300) % 4 == f
            t += float(rng.exponential(1.0 / (rate_burst if burst else rate_quiet)))
            size = int(min(max(rng.lognormal(np.log(med), 0.6), 1 << 20), 1 << 30))
            events.append((t, f, size, int(rng.integers(1, 5 if burst else 2))))
    events.sort()
    return events


def result_sizes(rng, n, median, sigma, lo, hi):
    """n lognormal result sizes around `median`, clipped to [lo, hi]."""
    return [int(min(max(rng.lognormal(np.log(median), sigma), lo), hi)) for _ in range(n)]


def two_stage_queue(sizes, capacity, lookahead, plan):
    """A two-stage workflow a -> b under memory pressure (the example of Sec. 7.2, at length), driven
    through a migration policy `plan(objects, capacity, incoming_bytes) -> (evict_ids, reload_ids)`.

    Request i's first stage a_i stores sizes[i] bytes; its second stage b_i consumes them. The a stages
    run `lookahead` requests ahead of the b stages: step i = a_{i+lookahead} stores its output (if there is
    such a request), then b_i runs and its data is dropped. `objects` is a list of
    dict(id, bytes, queue_pos, resident). Counts the b stages that found their input on the host (a reload
    on the critical path) and the bytes moved out and back. Returns dict(stalls, bytes_out, bytes_in)."""
    n = len(sizes)
    objs = {}
    stalls = bytes_out = bytes_in = 0

    def view(head):
        return [dict(id=i, bytes=o["bytes"], queue_pos=i - head, resident=o["resident"]) for i, o in sorted(objs.items())]

    def apply(evict, reload):
        nonlocal bytes_out, bytes_in
        for i in evict:
            objs[i]["resident"] = False
            bytes_out += objs[i]["bytes"]
        for i in reload:
            objs[i]["resident"] = True
            bytes_in += objs[i]["bytes"]

    for i in range(min(lookahead, n)):           # the a stages that are ahead at the start
        ev, rl = plan(view(0), capacity, sizes[i])
        apply(ev, [])
        objs[i] = {"bytes": sizes[i], "resident": True}
    for head in range(n):
        j = head + lookahead
        if j < n:
            ev, rl = plan(view(head), capacity, sizes[j])
            apply(ev, [])
            objs[j] = {"bytes": sizes[j], "resident": True}
        if not objs[head]["resident"]:           # b_head needs its input now
            stalls += 1
            ev, _ = plan([o for o in view(head) if o["id"] != head], capacity, sizes[head])
            apply(ev, [head])
        del objs[head]                           # consumed: cleared at once
        ev, rl = plan(view(head + 1), capacity, 0)
        apply(ev, rl)
    return {"stalls": stalls, "bytes_out": bytes_out, "bytes_in": bytes_in}


def hybrid_cube_mesh_24_48():
    """8 GPUs in a hybrid cube mesh, links of 24 or 48 GB/s per direction (one or two bricks), 6 bricks per
    GPU: a synthetic stand-in for the server of the paper's experiments (the text gives only the two link
    speeds and the non-uniformity). Returns the bandwidth matrix."""
    n = 8
    t = [[0] * n for _ in range(n)]
    for (a, b) in [(0, 3), (1, 2), (4, 7), (5, 6), (0, 4), (1, 5), (2, 6), (3, 7)]:
        t[a][b] = t[b][a] = 48
    for (a, b) in [(0, 1), (0, 2), (1, 3), (2, 3), (4, 5), (4, 6), (5, 7), (6, 7)]:
        t[a][b] = t[b][a] = 24
    return t


def full_mesh(n=8, bw=64):
    """Every GPU linked to every other by one link of `bw` GB/s (nodes with point-to-point links, 7 per GPU)."""
    return [[0 if a == b else bw for b in range(n)] for a in range(n)]
