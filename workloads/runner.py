"""Drive an engine (the CPU oracle or the HIP binding's harness) through a Plan.

An engine is any object with the calls
    host_arena(nbytes), pool_create(nbytes, slab_bytes), pool_grow(nbytes),
    slab_alloc(nbytes) -> offset, slab_free(offset),
    write_host(off, u8 array), read_host(off, n), write_pool(off, u8 array),
    read_pool(off, n), submit(descs, weights, chunk_bytes, flags) -> job,
    wait(job)
where a failing call raises an exception carrying ``.code``. Host addresses in
descriptors are offsets into the host arena. Nothing here computes a chunk, a
schedule or a copy.
"""
from dataclasses import dataclass, field

from .configs import seeded_bytes
from .format import FT_ENOMEM, FT_HOST, FT_POOL, make_descs


@dataclass
class RunRecord:
    alloc_off: dict = field(default_factory=dict)     # alloc id -> pool offset
    alloc_bytes: dict = field(default_factory=dict)
    jobs: dict = field(default_factory=dict)          # job name -> engine job handle
    descs: dict = field(default_factory=dict)         # job name -> DESC_DTYPE array
    weights: dict = field(default_factory=dict)
    chunk_bytes: dict = field(default_factory=dict)
    grows: list = field(default_factory=list)         # bytes of each appended segment
    pool_total: int = 0


def resolve(descs, alloc_off):
    out = []
    for d in descs:
        r = dict(d)
        for side in ("src", "dst"):
            ref = d[side]
            if ref[0] == "host":
                r[side + "_space"] = FT_HOST
                r[side] = ref[1]
            else:
                r[side + "_space"] = FT_POOL
                r[side] = alloc_off[ref[1]] + ref[2]
        out.append(r)
    return make_descs(out)


def run_plan(plan, engine, flags=0, fill=True, on_submit=None, do_wait=True):
    """Execute every step. ``fill`` False skips the (slow) seeded fills.
    ``on_submit(name, job)`` is called after each submit."""
    rec = RunRecord()
    engine.host_arena(plan.host_bytes)
    engine.pool_create(plan.pool_bytes, plan.slab_bytes)
    rec.pool_total = plan.pool_bytes
    targets = list(plan.grow_to)
    for st in plan.steps:
        op = st[0]
        if op == "alloc":
            _, aid, nbytes = st
            while True:
                try:
                    off = engine.slab_alloc(nbytes)
                    break
                except Exception as e:      # noqa: BLE001
                    if getattr(e, "code", None) != FT_ENOMEM or not targets:
                        raise
                    new_total = targets.pop(0)
                    engine.pool_grow(new_total - rec.pool_total)
                    rec.grows.append(new_total - rec.pool_total)
                    rec.pool_total = new_total
            rec.alloc_off[aid] = off
            rec.alloc_bytes[aid] = nbytes
        elif op == "fill_pool":
            _, aid, off, nbytes, seed = st
            if fill:
                engine.write_pool(rec.alloc_off[aid] + off, seeded_bytes(seed, nbytes))
        elif op == "fill_host":
            _, off, nbytes, seed = st
            if fill:
                engine.write_host(off, seeded_bytes(seed, nbytes))
        elif op == "submit":
            _, name, descs, weights, chunk_bytes = st
            arr = resolve(descs, rec.alloc_off)
            rec.descs[name] = arr
            rec.weights[name] = list(weights)
            rec.chunk_bytes[name] = chunk_bytes
            rec.jobs[name] = engine.submit(arr, list(weights), chunk_bytes, flags)
            if on_submit is not None:
                on_submit(name, rec.jobs[name])
        elif op == "wait":
            if do_wait:
                engine.wait(rec.jobs[st[1]])
        else:
            raise ValueError(op)
    return rec
