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
    """The two-stage workflow of Sec. 7.2 under memory pressure, run through `policy` (one of the two plans
    above). The workflow itself - who stores what when, who consumes it - is an input and lives with the other
    synthetic inputs (workloads.traces.two_stage_queue); the decisions are this module's."""
    from workloads.traces import two_stage_queue
    return two_stage_queue(sizes, capacity, lookahead, policy)


class Store:
    """The store of Sec. 7.2 over any engine object (slab_alloc / slab_free / submit / wait): results
    wait in the pool under a byte budget; the queue-aware rule above decides what moves to host memory
    and back, each move being one pool->host or host->pool transfer. The spill arena is a first-fit
    allocator in units of 4096 bytes over [spill_off, spill_off + spill_bytes) of the engine's host
    arena. Operations and their order of effects:

      put(id, nbytes, queue_pos)  evictions named by plan_queue_aware(objects, capacity, nbytes), in its
                                  order; then the allocation. Returns the pool offset.
      get(id)                     if the result is out: evictions named by the plan over the other
                                  objects with its bytes incoming, then it is brought back (a stall).
                                  Returns (offset, was_out).
      done(id)                    the result is dropped; then plan(objects, capacity, 0): evictions (none
                                  unless the budget was passed) and reloads in its order, a reload that
                                  finds no run of free slabs ends them.
      advance(steps)              every queue_pos decreases by steps, not below 0.
    """

    def __init__(self, engine, spill_off, spill_bytes, capacity, chunk_bytes, make_descs, host_space, pool_space):
        self.eng = engine
        self.spill_off, self.capacity, self.chunk = spill_off, capacity, chunk_bytes
        self.units = [False] * (spill_bytes // 4096)
        self.objs = {}
        self.make_descs, self.HOST, self.POOL = make_descs, host_space, pool_space
        self.log = []
        self.stalls = 0

    def _spill_alloc(self, nbytes):
        need = -(-nbytes // 4096)
        run = 0
        for i, used in enumerate(self.units):
            run = 0 if used else run + 1
            if run == need:
                first = i - need + 1
                for j in range(first, i + 1):
                    self.units[j] = True
                return first * 4096
        raise MemoryError("spill arena full")

    def _spill_free(self, at, nbytes):
        for j in range(at // 4096, at // 4096 + -(-nbytes // 4096)):
            self.units[j] = False

    def _move(self, src_space, src, dst_space, dst, n):
        d = self.make_descs([dict(func=0, src_space=src_space, dst_space=dst_space, src=src, dst=dst, row_bytes=n)])
        self.eng.wait(self.eng.submit(d, [1], self.chunk))

    def _view(self, skip=None):
        return [dict(id=i, bytes=o["bytes"], queue_pos=o["queue_pos"], resident=o["resident"])
                for i, o in sorted(self.objs.items()) if i != skip]

    def _out(self, i):
        o = self.objs[i]
        o["spill"] = self._spill_alloc(o["bytes"])
        self._move(self.POOL, o["off"], self.HOST, self.spill_off + o["spill"], o["bytes"])
        self.eng.slab_free(o["off"])
        o["resident"] = False
        self.log.append(("out", i))

    def _in(self, i):
        o = self.objs[i]
        o["off"] = self.eng.slab_alloc(o["bytes"])
        self._move(self.HOST, self.spill_off + o["spill"], self.POOL, o["off"], o["bytes"])
        self._spill_free(o["spill"], o["bytes"])
        o["resident"] = True
        self.log.append(("in", i, o["off"]))

    def put(self, i, nbytes, queue_pos):
        assert i not in self.objs and 0 < nbytes <= self.capacity
        evict, _ = plan_queue_aware(self._view(), self.capacity, nbytes)
        for e in evict:
            self._out(e)
        off = self.eng.slab_alloc(nbytes)
        self.objs[i] = dict(bytes=nbytes, queue_pos=queue_pos, resident=True, off=off)
        self.log.append(("put", i, off))
        return off

    def get(self, i):
        o = self.objs[i]
        was_out = not o["resident"]
        if was_out:
            evict, _ = plan_queue_aware(self._view(skip=i), self.capacity, o["bytes"])
            for e in evict:
                self._out(e)
            self._in(i)
            self.stalls += 1
        return o["off"], was_out

    def done(self, i):
        o = self.objs.pop(i)
        assert o["resident"]
        self.eng.slab_free(o["off"])
        evict, reload = plan_queue_aware(self._view(), self.capacity, 0)
        for e in evict:
            self._out(e)
        for r in reload:
            try:
                self._in(r)
            except Exception as e:      # noqa: BLE001  (the engine's "no run of free slabs")
                if getattr(e, "code", None) != -2:
                    raise
                break

    def advance(self, steps):
        for o in self.objs.values():
            o["queue_pos"] = max(o["queue_pos"] - steps, 0)

    def resident_bytes(self):
        return sum(o["bytes"] for o in self.objs.values() if o["resident"])
