"""Pins for the oracle's data result (Sec. 5.1: passing is a copy) and checks."""
import random

import numpy as np
import pytest

from oracle import (OracleEngine, OracleError, EINVAL, ERANGE, EOVERLAP, EBUSY,
                    H2P, P2H, P2P)
from oracle.engine import find_overlap
from workloads import make_descs, FT_HOST, FT_POOL
from workloads import configs, runner


def _engine(host=1 << 16, pool=1 << 18, slab=1024, seed=0):
    e = OracleEngine()
    e.host_arena(host)
    e.pool_create(pool, slab)
    rng = np.random.default_rng(seed)
    e.write_host(0, rng.integers(0, 256, host, dtype=np.uint8))
    return e, rng


def _random_descs(rng, e, n, nfunc):
    """Random non-overlapping 1-D/2-D descriptors of all three classes."""
    recs = []
    pyr = random.Random(int(rng.integers(1 << 30)))
    host_dst_cur = 40000          # host destinations live above the sources
    for i in range(n):
        rows = pyr.choice([1, 1, 2, 3, 7])
        rb = pyr.randint(1, 300)
        sp = rb + pyr.randint(0, 40)
        dp = rb + pyr.randint(0, 40)
        ext_s = (rows - 1) * sp + rb
        ext_d = (rows - 1) * dp + rb
        cls = pyr.choice([H2P, P2H, P2P])
        if cls == H2P:
            src = (FT_HOST, pyr.randint(0, 30000))
            a = e.slab_alloc(ext_d + 20)
            dst = (FT_POOL, a + pyr.randint(0, 19))
        elif cls == P2H:
            a = e.slab_alloc(ext_s + 20)
            e.write_pool(a, rng.integers(0, 256, ext_s + 20, dtype=np.uint8))
            src = (FT_POOL, a + pyr.randint(0, 19))
            dst = (FT_HOST, host_dst_cur + pyr.randint(0, 7))
            host_dst_cur += ext_d + 16
        else:
            a = e.slab_alloc(ext_s + 20)
            e.write_pool(a, rng.integers(0, 256, ext_s + 20, dtype=np.uint8))
            b = e.slab_alloc(ext_d + 20)
            src = (FT_POOL, a + pyr.randint(0, 19))
            dst = (FT_POOL, b + pyr.randint(0, 19))
        recs.append(dict(func=pyr.randrange(nfunc), src_space=src[0], src=src[1],
                         dst_space=dst[0], dst=dst[1], row_bytes=rb, rows=rows,
                         src_pitch=sp, dst_pitch=dp))
    return make_descs(recs)


def _byte_loop(e_host, e_pool, descs):
    """The formula dst[d.dst + r*dp + c] = src[d.src + r*sp + c], one byte at a time."""
    host = e_host.copy()
    pool = e_pool.copy()
    mem = {FT_HOST: host, FT_POOL: pool}
    src_host, src_pool = e_host, e_pool
    smem = {FT_HOST: src_host, FT_POOL: src_pool}
    for d in descs:
        for p in range(int(d["rows"]) * int(d["row_bytes"])):
            r, c = divmod(p, int(d["row_bytes"]))
            mem[int(d["dst_space"])][int(d["dst"]) + r * int(d["dst_pitch"]) + c] = \
                smem[int(d["src_space"])][int(d["src"]) + r * int(d["src_pitch"]) + c]
    return host, pool


def test_chunked_mover_equals_byte_loop_and_touches_nothing_else():
    for seed in range(12):
        e, rng = _engine(seed=seed)
        descs = _random_descs(rng, e, 14, nfunc=3)
        host0, pool0 = e.host_mem.copy(), e.pool_mem.copy()
        want_host, want_pool = _byte_loop(host0, pool0, descs)
        C = 16 * int(rng.integers(1, 20))
        w = [int(x) for x in rng.integers(1, 5, 3)]
        e.wait(e.submit(descs, w, C))
        assert np.array_equal(e.host_mem, want_host)
        assert np.array_equal(e.pool_mem, want_pool)


def test_chunked_mover_equals_definition():
    for seed in range(6):
        e, rng = _engine(seed=100 + seed)
        descs = _random_descs(rng, e, 20, nfunc=4)
        e2 = OracleEngine()
        e2.host_mem = e.host_mem.copy()
        e2.pool_mem = e.pool_mem.copy()
        e.wait(e.submit(descs, [1, 2, 3, 4], 64))
        e2.apply_definition(descs)
        assert np.array_equal(e.host_mem, e2.host_mem)
        assert np.array_equal(e.pool_mem, e2.pool_mem)


def test_one_d_is_memcpy_and_two_d_is_a_strided_view():
    e, rng = _engine()
    a = e.slab_alloc(5000)
    b = e.slab_alloc(64 * 50)
    src = bytes(e.host_mem[123:123 + 4321])
    d = make_descs([
        dict(func=0, src_space=FT_HOST, dst_space=FT_POOL, src=123, dst=a + 7, row_bytes=4321),
        dict(func=0, src_space=FT_HOST, dst_space=FT_POOL, src=9000, dst=b + 3, row_bytes=33,
             rows=40, src_pitch=100, dst_pitch=64)])
    view = np.lib.stride_tricks.as_strided(e.host_mem[9000:], shape=(40, 33), strides=(100, 1)).copy()
    e.wait(e.submit(d, [1], 256))
    assert bytes(e.pool_mem[a + 7:a + 7 + 4321]) == src
    got = np.lib.stride_tricks.as_strided(e.pool_mem[b + 3:], shape=(40, 33), strides=(64, 1))
    assert np.array_equal(got, view)
    # the gaps between destination rows keep the canary
    gaps = np.lib.stride_tricks.as_strided(e.pool_mem[b + 3 + 33:], shape=(39, 31), strides=(64, 1))
    assert np.all(gaps == 0xA5)


def test_result_does_not_depend_on_chunk_size_or_weights():
    images = []
    for C, w in ((16, [1, 1]), (4096, [5, 1]), (1 << 20, [1, 7])):
        e, rng = _engine(seed=42)
        descs = _random_descs(rng, e, 10, nfunc=2)
        e.wait(e.submit(descs, w, C))
        images.append((e.host_mem.copy(), e.pool_mem.copy()))
    for h, p in images[1:]:
        assert np.array_equal(h, images[0][0]) and np.array_equal(p, images[0][1])


def test_classes_are_scheduled_independently():
    e, rng = _engine()
    a = e.slab_alloc(1000)
    b = e.slab_alloc(1000)
    c = e.slab_alloc(1000)
    d = make_descs([
        dict(func=0, src_space=FT_HOST, dst_space=FT_POOL, src=0, dst=a, row_bytes=100),
        dict(func=1, src_space=FT_POOL, dst_space=FT_POOL, src=b, dst=c, row_bytes=40),
        dict(func=1, src_space=FT_HOST, dst_space=FT_POOL, src=500, dst=a + 200, row_bytes=20),
        dict(func=0, src_space=FT_POOL, dst_space=FT_HOST, src=b + 100, dst=50000, row_bytes=16)])
    j = e.submit(d, [1, 1], 32)
    assert e.job_schedule(j, H2P) == [(0, 0), (1, 0), (0, 1), (0, 2), (0, 3)]
    assert e.job_schedule(j, P2P) == [(1, 0), (1, 1)]
    assert e.job_schedule(j, P2H) == [(0, 0)]


def _brute_overlap(descs):
    for space in (FT_HOST, FT_POOL):
        dst_count = {}
        srcs = set()
        for d in descs:
            for r in range(int(d["rows"])):
                for c in range(int(d["row_bytes"])):
                    if int(d["dst_space"]) == space:
                        a = int(d["dst"]) + r * int(d["dst_pitch"]) + c
                        dst_count[a] = dst_count.get(a, 0) + 1
                    if int(d["src_space"]) == space:
                        srcs.add(int(d["src"]) + r * int(d["src_pitch"]) + c)
        if any(v > 1 for v in dst_count.values()) or (srcs & set(dst_count)):
            return True
    return False


def test_overlap_checker_against_byte_marking():
    pyr = random.Random(9)
    hits = 0
    for _ in range(600):
        recs = []
        for _ in range(pyr.randint(1, 4)):
            rows = pyr.choice([1, 2, 3])
            rb = pyr.randint(1, 12)
            recs.append(dict(func=0, src_space=pyr.choice([FT_HOST, FT_POOL]), dst_space=FT_POOL,
                             src=pyr.randint(0, 60), dst=pyr.randint(0, 60), row_bytes=rb, rows=rows,
                             src_pitch=rb + pyr.randint(0, 6), dst_pitch=rb + pyr.randint(0, 6)))
        d = make_descs(recs)
        want = _brute_overlap(d)
        hits += want
        assert find_overlap(d) == want
    assert 100 < hits < 500     # both outcomes are exercised


def test_error_codes():
    e, _ = _engine()
    a = e.slab_alloc(2048)
    good = dict(func=0, src_space=FT_HOST, dst_space=FT_POOL, src=0, dst=a, row_bytes=100)

    def code(descs, w=(1,), C=64):
        with pytest.raises(OracleError) as ei:
            e.submit(make_descs(descs), list(w), C)
        return ei.value.code

    assert code([good], w=()) == EINVAL
    assert code([good], w=(0,)) == EINVAL
    assert code([good], C=0) == EINVAL
    assert code([good], C=24) == EINVAL
    assert code([dict(good, func=1)]) == EINVAL
    assert code([dict(good, flags=1)]) == EINVAL
    assert code([dict(good, dst_space=FT_HOST)]) == EINVAL          # host -> host
    assert code([dict(good, row_bytes=0)]) == EINVAL
    assert code([dict(good, rows=0)]) == EINVAL
    assert code([dict(good, rows=2, src_pitch=99, dst_pitch=100)]) == EINVAL
    assert code([dict(good, rows=2, src_pitch=100, dst_pitch=99)]) == EINVAL
    assert code([dict(good, dst=a + 2048 - 99)]) == ERANGE           # runs off the allocation
    assert code([dict(good, dst=a + 4096)]) == ERANGE                # not allocated at all
    assert code([dict(good, rows=3, src_pitch=100, dst_pitch=1000)]) == ERANGE
    assert code([dict(good, src=(1 << 16) - 50)]) == ERANGE          # past the host arena
    assert code([good, dict(good, src=200, dst=a + 99)]) == EOVERLAP
    assert code([dict(good, src_space=FT_POOL, src=a + 50)]) == EOVERLAP   # dst also read
    # nothing moved by any of the rejected submits
    assert np.all(e.pool_mem == 0xA5)
    # EINVAL is reported before ERANGE, ERANGE before EOVERLAP
    assert code([dict(good, dst=a + 4096), dict(good, row_bytes=0)]) == EINVAL
    assert code([good, dict(good, src=200, dst=a + 99), dict(good, dst=a + 4096)]) == ERANGE


def test_empty_submit_and_busy_free():
    e, _ = _engine()
    j = e.submit(make_descs([]), [1], 64)
    e.wait(j)
    a = e.slab_alloc(100)
    j = e.submit(make_descs([dict(func=0, src_space=FT_HOST, dst_space=FT_POOL, src=0, dst=a,
                                  row_bytes=10)]), [1], 64)
    with pytest.raises(OracleError) as ei:
        e.slab_free(a)
    assert ei.value.code == EBUSY
    e.wait(j)
    e.slab_free(a)
    with pytest.raises(OracleError) as ei:
        e.wait(j)
    assert ei.value.code == EINVAL


@pytest.mark.parametrize("name,scale", [("tiny", 0.05), ("traffic", 0.13), ("feature", 0.002),
                                        ("contended", 0.004), ("large_mixed", 0.002)])
def test_workloads_round_trip_through_definition(name, scale):
    """Every config: the chunked result equals the plain definition applied to a
    second image, and every destination equals its seeded source."""
    plan = configs.CONFIGS[name](scale)
    e = OracleEngine()
    rec = runner.run_plan(plan, e)
    e2 = OracleEngine()

    class Plain(OracleEngine):
        def submit(self, descs, weights, chunk_bytes, flags=0):
            self._check(descs, weights, chunk_bytes)
            self.apply_definition(descs)
            self.jobs[self._next_job] = type("J", (), {"pending": True, "allocs": set()})()
            self._next_job += 1
            return self._next_job - 1

    e2 = Plain()
    rec2 = runner.run_plan(plan, e2)
    assert rec.alloc_off == rec2.alloc_off
    assert np.array_equal(e.host_mem, e2.host_mem)
    assert np.array_equal(e.pool_mem, e2.pool_mem)
    moved = sum(int(d["rows"]) * int(d["row_bytes"]) for arr in rec.descs.values() for d in arr)
    assert moved == plan.payload_bytes()


def test_pageable_source_is_a_plain_copy():
    """Sec. 6.1's circular pinned buffer is transport: a source in ordinary host memory gives the
    same result as any other copy (NumPy slicing), chunked or not; host to host stays invalid."""
    import oracle
    from oracle import OracleEngine, OracleError
    from workloads import make_descs
    rng = np.random.default_rng(77)
    eng = OracleEngine()
    eng.host_arena(1 << 16)
    eng.pageable_arena(1 << 18)
    eng.pool_create(1 << 20, 4096)
    data = rng.integers(0, 256, 1 << 18, dtype=np.uint8)
    eng.write_pageable(0, data)
    a = eng.slab_alloc(100000)
    b = eng.slab_alloc(64 * 300)
    recs = [dict(func=0, src_space=oracle.PAGEABLE, dst_space=oracle.POOL, src=12345, dst=a + 7, row_bytes=90001),
            dict(func=1, src_space=oracle.PAGEABLE, dst_space=oracle.POOL, src=150000, dst=b, row_bytes=64, rows=300,
                 src_pitch=200, dst_pitch=64)]
    before = eng.pool_mem.copy()
    eng.wait(eng.submit(make_descs(recs), [1, 3], 4096))
    want = before
    want[a + 7:a + 7 + 90001] = data[12345:12345 + 90001]
    rows = np.lib.stride_tricks.as_strided(data[150000:], shape=(300, 64), strides=(200, 1))
    want[b:b + 64 * 300] = rows.reshape(-1)
    assert np.array_equal(eng.pool_mem, want)
    assert oracle.link_class(oracle.PAGEABLE, oracle.POOL) == oracle.H2P
    for bad in (dict(func=0, src_space=oracle.PAGEABLE, dst_space=oracle.HOST, src=0, dst=0, row_bytes=16),
                dict(func=0, src_space=oracle.HOST, dst_space=oracle.PAGEABLE, src=0, dst=0, row_bytes=16),
                dict(func=0, src_space=oracle.PAGEABLE, dst_space=oracle.PAGEABLE, src=0, dst=64, row_bytes=16)):
        with pytest.raises(OracleError) as ei:
            eng.submit(make_descs([bad]), [1], 4096)
        assert ei.value.code == oracle.EINVAL
    with pytest.raises(OracleError) as ei:
        eng.submit(make_descs([dict(func=0, src_space=oracle.PAGEABLE, dst_space=oracle.POOL, src=(1 << 18) - 8, dst=a,
                                    row_bytes=16)]), [1], 4096)
    assert ei.value.code == oracle.ERANGE


def test_pageable_destination_is_a_plain_copy():
    """The other direction of the host link through the same buffer (Sec. 6.1 names the buffer for PCIe
    transfers as such): pool -> ordinary host memory is the plain copy too, nothing else in that memory
    changes, it is a pool->host transfer for the schedule, and aliasing inside it is still refused."""
    import oracle
    from oracle import OracleEngine, OracleError
    from workloads import make_descs
    rng = np.random.default_rng(78)
    eng = OracleEngine()
    eng.host_arena(1 << 16)
    eng.pageable_arena(1 << 18, fill=0x3C)
    eng.pool_create(1 << 20, 4096)
    a = eng.slab_alloc(120000)
    b = eng.slab_alloc(50 * 333)
    data = rng.integers(0, 256, 120000, dtype=np.uint8)
    rowsrc = rng.integers(0, 256, 50 * 333, dtype=np.uint8)
    eng.write_pool(a, data)
    eng.write_pool(b, rowsrc)
    recs = [dict(func=0, src_space=oracle.POOL, dst_space=oracle.PAGEABLE, src=a + 3, dst=1001, row_bytes=100003),
            dict(func=1, src_space=oracle.POOL, dst_space=oracle.PAGEABLE, src=b, dst=150001, row_bytes=50, rows=333,
                 src_pitch=50, dst_pitch=77),
            dict(func=1, src_space=oracle.POOL, dst_space=oracle.HOST, src=a, dst=5, row_bytes=999)]
    pool_before, host_before = eng.pool_mem.copy(), eng.host_mem.copy()
    job = eng.submit(make_descs(recs), [2, 1], 4096)
    eng.wait(job)
    want = np.full(1 << 18, 0x3C, dtype=np.uint8)
    want[1001:1001 + 100003] = data[3:3 + 100003]
    for r in range(333):
        want[150001 + 77 * r:150001 + 77 * r + 50] = rowsrc[50 * r:50 * r + 50]
    assert np.array_equal(eng.pageable_mem, want)
    assert np.array_equal(eng.pool_mem, pool_before)
    host_before[5:5 + 999] = data[:999]
    assert np.array_equal(eng.host_mem, host_before)
    assert oracle.link_class(oracle.POOL, oracle.PAGEABLE) == oracle.P2H
    assert eng.job_class_bytes(job, oracle.P2H) == 100003 + 50 * 333 + 999
    assert len(eng.job_schedule(job, oracle.P2H)) == -(-100003 // 4096) + -(-(50 * 333 + 999) // 4096)
    twice = [dict(func=0, src_space=oracle.POOL, dst_space=oracle.PAGEABLE, src=a, dst=100, row_bytes=64),
             dict(func=0, src_space=oracle.POOL, dst_space=oracle.PAGEABLE, src=a + 64, dst=163, row_bytes=64)]
    with pytest.raises(OracleError) as ei:
        eng.submit(make_descs(twice), [1], 4096)
    assert ei.value.code == oracle.EOVERLAP
    with pytest.raises(OracleError) as ei:
        eng.submit(make_descs([dict(func=0, src_space=oracle.POOL, dst_space=oracle.PAGEABLE, src=a, dst=(1 << 18) - 8,
                                    row_bytes=16)]), [1], 4096)
    assert ei.value.code == oracle.ERANGE
