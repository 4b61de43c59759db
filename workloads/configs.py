"""The five seeded transfer mixes, as pure data.

Each builder returns a ``Plan``: the pool geometry, the size of the host arena
and a list of steps (allocate, fill, submit, wait) whose descriptors still
refer to allocations by id. ``runner.run_plan`` resolves the ids with the
offsets an engine hands out. Shapes follow the inference workflows the paper
evaluates (video frames fanned out to recognisers, feature maps passed
between GPU functions, several functions sharing the host link); the paper's
datasets and traces are not used, only shapes and sizes.

``scale`` < 1 shrinks byte sizes (never the structure) so that the CPU oracle
finishes in seconds; scale = 1 is the full configuration.
"""
from dataclasses import dataclass, field

import numpy as np

from .format import FT_HOST, FT_POOL

BASE_SEED = 241101830
MiB = 1 << 20
KiB = 1 << 10


def seeded_bytes(seed, nbytes):
    """nbytes of incompressible bytes from PCG64(seed)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    words = rng.integers(0, 1 << 64, size=(nbytes + 7) // 8, dtype=np.uint64)
    return words.view(np.uint8)[:nbytes]


def _up(x, a):
    return -(-x // a) * a


@dataclass
class Plan:
    name: str
    slab_bytes: int
    pool_bytes: int                 # first segment
    host_bytes: int
    grow_to: list = field(default_factory=list)   # total pool sizes to grow through on ENOMEM
    steps: list = field(default_factory=list)
    # step forms:
    #   ("alloc", id, nbytes)
    #   ("fill_pool", id, offset, nbytes, seed)
    #   ("fill_host", offset, nbytes, seed)
    #   ("submit", job_name, descs, weights, chunk_bytes)    descs: list of dicts, see below
    #   ("wait", job_name)
    # a descriptor dict has func,row_bytes,rows,src_pitch,dst_pitch and
    #   src / dst = ("host", offset) or ("pool", alloc_id, offset)

    def payload_bytes(self):
        tot = 0
        for st in self.steps:
            if st[0] == "submit":
                tot += sum(d["row_bytes"] * d.get("rows", 1) for d in st[2])
        return tot


def _d1(func, src, dst, nbytes):
    return dict(func=func, src=src, dst=dst, row_bytes=nbytes, rows=1,
                src_pitch=nbytes, dst_pitch=nbytes)


def tiny(scale=1.0, seed=BASE_SEED + 1):
    """4 equal-weight functions, 8 tensors each, host->pool then pool->host."""
    rng = np.random.Generator(np.random.PCG64(seed))
    F, per = 4, 8
    hi = max(8 * KiB, int(1 * MiB * scale))
    sizes = rng.integers(4 * KiB, hi + 1, size=F * per)
    plan = Plan("tiny", slab_bytes=256 * KiB, pool_bytes=64 * MiB, host_bytes=0)
    src_off, dst_off = [], []
    cur = 0
    for n in sizes:                     # sources, each in its own 4 KiB-aligned window
        src_off.append(cur)
        cur = _up(cur + int(n), 4 * KiB)
    for n in sizes:                     # pool->host destinations
        dst_off.append(cur)
        cur = _up(cur + int(n), 4 * KiB)
    plan.host_bytes = cur
    a_descs, b_descs = [], []
    for i, n in enumerate(sizes):
        n = int(n)
        f = i // per
        plan.steps.append(("alloc", i, n))
        plan.steps.append(("fill_host", src_off[i], n, seed * 1000 + i))
        a_descs.append(_d1(f, ("host", src_off[i]), ("pool", i, 0), n))
        b_descs.append(_d1(f, ("pool", i, 0), ("host", dst_off[i]), n))
    w = [1, 1, 1, 1]
    plan.steps += [("submit", "h2p", a_descs, w, 64 * KiB), ("wait", "h2p"),
                   ("submit", "p2h", b_descs, w, 64 * KiB), ("wait", "p2h")]
    return plan


def traffic(scale=1.0, seed=BASE_SEED + 2):
    """16 decoded frames host->pool, then 32 crops per frame gathered
    pool->pool into two recognisers' buffers (weights 1:1)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    nframes = 16 if scale >= 1.0 else max(2, int(16 * scale))
    ncrops = 32 if scale >= 1.0 else max(4, int(32 * scale))
    CH, FH, FW = 3, 1080, 1920
    frame_bytes = CH * FH * FW
    plan = Plan("traffic", slab_bytes=1 * MiB, pool_bytes=0, host_bytes=nframes * _up(frame_bytes, 4 * KiB))
    a_descs = []
    for i in range(nframes):
        hoff = i * _up(frame_bytes, 4 * KiB)
        plan.steps.append(("alloc", i, frame_bytes))
        plan.steps.append(("fill_host", hoff, frame_bytes, seed * 1000 + i))
        a_descs.append(_d1(0, ("host", hoff), ("pool", i, 0), frame_bytes))
    crops = []
    run = [0, 0]
    for i in range(nframes):
        for _ in range(ncrops):
            h = int(rng.integers(64, 257))
            w = int(rng.integers(64, 257))
            y = int(rng.integers(0, FH - h + 1))
            x = int(rng.integers(0, FW - w + 1))
            c = int(rng.integers(0, 2))
            crops.append((i, h, w, y, x, c, run[c]))
            run[c] = _up(run[c] + CH * h * w, 16)
    rec_id = [nframes, nframes + 1]
    for c in (0, 1):
        plan.steps.append(("alloc", rec_id[c], max(run[c], 16)))
    b_descs = []
    for (i, h, w, y, x, c, doff) in crops:
        for ch in range(CH):
            b_descs.append(dict(func=c, rows=h, row_bytes=w, src_pitch=FW, dst_pitch=w,
                                src=("pool", i, ch * FH * FW + y * FW + x),
                                dst=("pool", rec_id[c], doff + ch * h * w)))
    slabs = sum(_up(frame_bytes, MiB) for _ in range(nframes)) + sum(_up(max(r, 16), MiB) for r in run)
    plan.pool_bytes = slabs + 4 * MiB
    # both jobs go to one stream, which runs them in submit order: the crops job reads
    # the frames only after they have landed, with no host wait in between
    plan.steps += [("submit", "frames", a_descs, [1], 2 * MiB),
                   ("submit", "crops", b_descs, [1, 1], 256 * KiB),
                   ("wait", "frames"), ("wait", "crops")]
    return plan


FEATURE_WEIGHTS = [1, 1, 2, 2, 4, 4, 8, 8]


def feature(scale=1.0, seed=BASE_SEED + 3):
    """64 fp16 feature maps passed pool->pool between 8 functions, weights 1:1:2:2:4:4:8:8."""
    rng = np.random.Generator(np.random.PCG64(seed))
    n = 64
    B = rng.choice([1, 8, 32], size=n)
    C = rng.choice([64, 256, 512], size=n)
    H = rng.choice([14, 28, 56], size=n)
    sizes = [int(2 * b * c * h * h) for b, c, h in zip(B, C, H)]
    if scale < 1.0:
        sizes = [max(25088, _up(int(s * scale), 16)) for s in sizes]
    plan = Plan("feature", slab_bytes=1 * MiB, pool_bytes=0, host_bytes=4 * KiB)
    descs = []
    for i, s in enumerate(sizes):
        plan.steps.append(("alloc", i, s))
        plan.steps.append(("fill_pool", i, 0, s, seed * 1000 + i))
    for i, s in enumerate(sizes):
        plan.steps.append(("alloc", n + i, s))
        descs.append(_d1(i % 8, ("pool", i, 0), ("pool", n + i, 0), s))
    need = 2 * sum(_up(s, MiB) for s in sizes)
    plan.pool_bytes = _up(need + need // 10, MiB)
    plan.steps += [("submit", "pass", descs, list(FEATURE_WEIGHTS), 2 * MiB), ("wait", "pass")]
    return plan


def contended(scale=1.0, seed=BASE_SEED + 4):
    """16 functions each streaming one large buffer host->pool, weights from {1,2,4}."""
    rng = np.random.Generator(np.random.PCG64(seed))
    F = 16
    per = _up(max(1 * MiB + 4 * KiB, int(256 * MiB * scale)), 16)
    arena = _up(max(4 * per, int(1024 * MiB * scale)), 4 * KiB)
    w = [int(x) for x in rng.choice([1, 2, 4], size=F)]
    plan = Plan("contended", slab_bytes=1 * MiB, pool_bytes=_up(F * _up(per, MiB) + 16 * MiB, MiB),
                host_bytes=arena)
    plan.steps.append(("fill_host", 0, arena, seed * 1000))
    offs = rng.choice((arena - per) // (4 * KiB) + 1, size=F, replace=False) * (4 * KiB)
    descs = []
    for f in range(F):
        plan.steps.append(("alloc", f, per))
        descs.append(_d1(f, ("host", int(offs[f])), ("pool", f, 0), per))
    plan.steps += [("submit", "stream", descs, w, 512 * KiB), ("wait", "stream")]
    return plan


def large_mixed(scale=1.0, seed=BASE_SEED + 5):
    """1024 transfers, lognormal sizes, 60% host->pool / 40% pool->pool, 10% at
    unaligned offsets, issued in 16 waves while the pool grows by doubling."""
    rng = np.random.Generator(np.random.PCG64(seed))
    n, F, waves = 1024, 16, 16
    total = int(8 * 1024 * MiB * scale)
    lo, hi = 4 * KiB, max(64 * KiB, int(256 * MiB * scale))
    med = max(16 * KiB, 2 * MiB * scale)
    raw = np.exp(rng.normal(np.log(med), 1.5, size=n))
    raw = np.clip(raw, lo, hi)
    for _ in range(8):                       # rescale to the target sum, re-clip
        raw = np.clip(raw * (total / raw.sum()), lo, hi)
    sizes = [int(x) for x in raw]
    unaligned = rng.random(n) < 0.10
    h2p = rng.random(n) < 0.60
    sizes = [s if u else _up(s, 16) for s, u in zip(sizes, unaligned)]
    w = [int(x) for x in rng.choice([1, 2, 4], size=F)]
    arena = _up(max(2 * hi, int(1024 * MiB * scale)), 4 * KiB)
    slab = 1 * MiB if scale >= 1.0 else 4 * KiB
    first = _up(int(1024 * MiB * scale), slab)
    plan = Plan("large_mixed", slab_bytes=slab, pool_bytes=first, host_bytes=arena,
                grow_to=[first * m for m in (2, 4, 8, 16, 32)])
    plan.steps.append(("fill_host", 0, arena, seed * 1000))
    per_wave = n // waves
    next_id = 0
    for wv in range(waves):
        descs = []
        for i in range(wv * per_wave, (wv + 1) * per_wave):
            s = sizes[i]
            so = int(rng.integers(1, 16)) if unaligned[i] else 0
            do = int(rng.integers(1, 16)) if unaligned[i] else 0
            dst_id = next_id
            next_id += 1
            plan.steps.append(("alloc", dst_id, s + 16))
            if h2p[i]:
                hoff = int(rng.integers(0, (arena - s - 16) // 16 + 1)) * 16 + so
                descs.append(_d1(i % F, ("host", hoff), ("pool", dst_id, do), s))
            else:
                src_id = next_id
                next_id += 1
                plan.steps.append(("alloc", src_id, s + 16))
                plan.steps.append(("fill_pool", src_id, 0, s + 16, seed * 1000 + 1 + i))
                descs.append(_d1(i % F, ("pool", src_id, so), ("pool", dst_id, do), s))
        plan.steps.append(("submit", f"wave{wv}", descs, w, 2 * MiB))
    for wv in range(waves):
        plan.steps.append(("wait", f"wave{wv}"))
    return plan


def first_submits(plan, count):
    """The same plan cut after its first `count` submits (a bounded sample of the workload)."""
    steps = []
    seen = 0
    names = []
    for st in plan.steps:
        if st[0] == "wait":
            continue
        steps.append(st)
        if st[0] == "submit":
            names.append(st[1])
            seen += 1
            if seen == count:
                break
    steps += [("wait", n) for n in names]
    return Plan(plan.name, plan.slab_bytes, plan.pool_bytes, plan.host_bytes, list(plan.grow_to), steps)


CONFIGS = {"tiny": tiny, "traffic": traffic, "feature": feature,
           "contended": contended, "large_mixed": large_mixed}
