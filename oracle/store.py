"""Elastic GPU data store of Sec. 7: how large the pool should be, and what to move
out of it (and back) under memory pressure.

Sec. 7.1 (auto-scaling pool). Per function three histograms are kept: the interval
between its requests, the size of its intermediate data, and how many of its results
are held at once. With R_window, R_size, R_con their 99th percentiles, each execution
of the function reserves R_size * R_con bytes for the next R_window seconds; a
reservation that sees no new request in its window is given back. The pool's size at
time t is the sum of the reservations whose window holds t, never below a floor
(300 MB in the paper's experiments).

Sec. 7.2 (queue-aware migration). When the store is over its capacity, the data to
move to host memory first is the data whose consumer is furthest back in the request
queue (not the least recently stored, which is usually the next to be needed);
data moved out is brought back, nearest consumer first, as soon as there is room.

Readings where the text is silent:
  * percentile: nearest rank, the ceil(q*n)-th smallest of the n samples;
  * a function with no interval sample yet (one request so far) gets `default_window`;
  * every observation refreshes the function's reservation (size and window) from the
    histograms as they stand after it;
  * eviction order: largest queue position first, ties to the larger object id (the
    later stored); reload order: smallest queue position first, ties to the smaller id;
    an object is reloaded only if it fits entirely; objects of the request at the head of
    the queue are reloaded before anything else is considered;
  * least-recently-stored eviction (the policy the paper argues against) is here too,
    as the yardstick.

TEST INFRASTRUCTURE ONLY (see the package docstring).
"""
import math


def percentile_nearest_rank(samples, q):
    if not samples:
        raise ValueError("no samples")
    s = sorted(samples)
    rank = int(math.ceil(q * len(s)))
    rank = min(max(rank, 1), len(s))
    return s[rank - 1]


class Sizer:
    def __init__(self, min_bytes, quantile=0.99, default_window=60.0):
        self.min_bytes = int(min_bytes)
        self.q = float(quantile)
        self.default_window = float(default_window)
        self.hist = {}     # func -> dict(last, intervals, sizes, cons)
        self.resv = {}     # func -> (bytes, expires)

    def observe(self, func, t, data_size, concurrency):
        h = self.hist.setdefault(func, {"last": None, "intervals": [], "sizes": [], "cons": []})
        if h["last"] is not None:
            h["intervals"].append(float(t) - h["last"])
        h["last"] = float(t)
        h["sizes"].append(int(data_size))
        h["cons"].append(int(concurrency))
        r_size = percentile_nearest_rank(h["sizes"], self.q)
        r_con = percentile_nearest_rank(h["cons"], self.q)
        r_window = percentile_nearest_rank(h["intervals"], self.q) if h["intervals"] else self.default_window
        self.resv[func] = (r_size * r_con, float(t) + r_window)

    def target(self, t):
        total = 0
        for nbytes, expires in self.resv.values():
            if float(t) <= expires:
                total += nbytes
        return max(total, self.min_bytes)


def plan_queue_aware(objects, capacity, incoming=0):
    """objects: list of dicts id, bytes, queue_pos, resident. Returns (evict ids in order,
    reload ids in order) so that resident bytes + incoming <= capacity after the evictions,
    and then whatever fits is brought back."""
    used = sum(o["bytes"] for o in objects if o["resident"]) + incoming
    evict = []
    for o in sorted((o for o in objects if o["resident"]), key=lambda o: (-o["queue_pos"], -o["id"])):
        if used <= capacity:
            break
        evict.append(o["id"])
        used -= o["bytes"]
    reload = []
    if not evict:
        for o in sorted((o for o in objects if not o["resident"]), key=lambda o: (o["queue_pos"], o["id"])):
            if used + o["bytes"] <= capacity:
                reload.append(o["id"])
                used += o["bytes"]
            else:
                break
    return evict, reload


def plan_lru(objects, capacity, incoming=0):
    """The same with least-recently-stored eviction (ids grow with store time) and reloads only on demand."""
    used = sum(o["bytes"] for o in objects if o["resident"]) + incoming
    evict = []
    for o in sorted((o for o in objects if o["resident"]), key=lambda o: o["id"]):
        if used <= capacity:
            break
        evict.append(o["id"])
        used -= o["bytes"]
    return evict, []


def simulate_queue(sizes, capacity, lookahead, policy):
    """A two-stage workflow a -> b under memory pressure (Sec. 7.2's example, at length).

    Request i's first stage a_i stores sizes[i] bytes; its second stage b_i consumes them.
    The a stages run `lookahead` requests ahead of the b stages: step i = a_{i+lookahead}
    stores its output (if there is such a request), then b_i runs and its data is dropped.
    Counts the b stages that found their input on the host (a reload on the critical
    path) and the bytes moved out and back. Returns dict(stalls, bytes_out, bytes_in)."""
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
        ev, rl = policy(view(0), capacity, sizes[i])
        apply(ev, [])
        objs[i] = {"bytes": sizes[i], "resident": True}
    for head in range(n):
        j = head + lookahead
        if j < n:
            ev, rl = policy(view(head), capacity, sizes[j])
            apply(ev, [])
            objs[j] = {"bytes": sizes[j], "resident": True}
        if not objs[head]["resident"]:           # b_head needs its input now
            stalls += 1
            ev, _ = policy([o for o in view(head) if o["id"] != head], capacity, sizes[head])
            apply(ev, [head])
        del objs[head]                           # consumed: cleared at once
        ev, rl = policy(view(head + 1), capacity, 0)
        apply(ev, rl)
    return {"stalls": stalls, "bytes_out": bytes_out, "bytes_in": bytes_in}
