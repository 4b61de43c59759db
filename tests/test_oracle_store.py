"""Pins of the oracle's Sec. 7 policies (pool sizing by histograms, queue-aware migration)
and the library's host-side versions held against them. No GPU."""
import random

import numpy as np
import pytest

from oracle import OracleError, EINVAL, EBUSY
from oracle.pool import Pool
from oracle.store import (Sizer, percentile_nearest_rank, plan_lru, plan_queue_aware, simulate_queue)


def test_percentile_is_numpys_inverted_cdf():
    rng = random.Random(2)
    for _ in range(300):
        n = rng.randint(1, 60)
        v = [rng.randint(0, 1000) for _ in range(n)]
        q = rng.choice([0.5, 0.9, 0.99, 1.0, 0.01])
        assert percentile_nearest_rank(v, q) == int(np.percentile(v, q * 100, method="inverted_cdf"))
    assert percentile_nearest_rank([5], 0.99) == 5
    assert percentile_nearest_rank(list(range(1, 101)), 0.99) == 99      # the 99th of 100
    assert percentile_nearest_rank(list(range(1, 201)), 0.99) == 198     # ceil(198.0)


def test_sizer_by_hand():
    # Sec. 7.1: reservation = R_size * R_con for R_window after each execution; sum over the
    # functions whose window holds t; never below the floor.
    s = Sizer(min_bytes=300, quantile=0.99, default_window=60.0)
    assert s.target(0.0) == 300
    s.observe(0, 0.0, 1000, 1)                  # first request: default window
    assert s.target(0.0) == 1000 and s.target(60.0) == 1000 and s.target(60.1) == 300
    s.observe(0, 10.0, 2000, 2)                 # interval 10 -> window 10; sizes {1000,2000}, cons {1,2}
    assert s.target(10.0) == 4000 and s.target(20.0) == 4000 and s.target(20.5) == 300
    s.observe(1, 15.0, 500, 4)                  # another function, alive 60 s
    assert s.target(15.0) == 4000 + 2000
    assert s.target(21.0) == 2000               # function 0 reclaimed, function 1 still reserved
    assert s.target(80.0) == 300
    # 99th percentile ignores one outlier in 200 samples but not in 50
    s = Sizer(0)
    for i in range(199):
        s.observe(0, float(i), 100, 1)
    s.observe(0, 199.0, 10**9, 1)
    assert s.target(199.0) == 100
    s = Sizer(0)
    for i in range(49):
        s.observe(0, float(i), 100, 1)
    s.observe(0, 49.0, 10**9, 1)
    assert s.target(49.0) == 10**9


def test_paper_example_queue_aware_moves_the_later_output_first():
    # Sec. 7.2 / its figure: outputs of a1 and a2 are stored, b1 is queued before b2. Under
    # pressure LRU moves a1's output (stored first) although b1 needs it next; the queue-aware
    # rule moves a2's output, and brings it back once a1's output has been consumed.
    objs = [dict(id=1, bytes=400, queue_pos=0, resident=True), dict(id=2, bytes=400, queue_pos=1, resident=True)]
    assert plan_queue_aware(objs, 1000, incoming=400) == ([2], [])
    assert plan_lru(objs, 1000, incoming=400) == ([1], [])
    after = [dict(id=2, bytes=400, queue_pos=0, resident=False), dict(id=3, bytes=400, queue_pos=1, resident=True)]
    assert plan_queue_aware(after, 1000) == ([], [2])


def test_plan_properties():
    rng = random.Random(8)
    for _ in range(500):
        n = rng.randint(0, 12)
        objs = [dict(id=i, bytes=rng.randint(1, 100), queue_pos=rng.randint(0, 6), resident=rng.random() < 0.6)
                for i in range(n)]
        cap, inc = rng.randint(0, 400), rng.randint(0, 100)
        ev, rl = plan_queue_aware(objs, cap, inc)
        by_id = {o["id"]: o for o in objs}
        assert all(by_id[i]["resident"] for i in ev) and all(not by_id[i]["resident"] for i in rl)
        assert len(set(ev)) == len(ev) and not (ev and rl)
        used = sum(o["bytes"] for o in objs if o["resident"]) + inc
        left = used - sum(by_id[i]["bytes"] for i in ev)
        assert left <= cap or all(not o["resident"] or o["id"] in ev for o in objs)
        if ev:    # no eviction more than needed: without the last one it would not fit
            assert left + by_id[ev[-1]]["bytes"] > cap
            # furthest consumers go first: nobody kept is further back than somebody moved
            kept = [o for o in objs if o["resident"] and o["id"] not in ev]
            assert all(k["queue_pos"] <= min(by_id[i]["queue_pos"] for i in ev) for k in kept)
        assert left + sum(by_id[i]["bytes"] for i in rl) <= max(cap, left)
        if rl:    # nearest consumers come back first
            assert [by_id[i]["queue_pos"] for i in rl] == sorted(by_id[i]["queue_pos"] for i in rl)


def test_queue_aware_never_stalls_more_than_lru():
    rng = random.Random(12)
    worse = 0
    for _ in range(60):
        n = rng.randint(20, 120)
        sizes = [rng.randint(20, 200) for _ in range(n)]
        cap = rng.randint(250, 1500)
        look = rng.randint(1, 15)
        qa = simulate_queue(sizes, cap, look, plan_queue_aware)
        lru = simulate_queue(sizes, cap, look, plan_lru)
        assert qa["stalls"] <= lru["stalls"]
        worse += lru["stalls"] > qa["stalls"]
        if sum(sorted(sizes)[-look - 1:]) <= cap:      # everything in flight always fits: nothing moves
            assert qa == {"stalls": 0, "bytes_out": 0, "bytes_in": 0} == lru
    assert worse > 20


def test_pool_shrink_against_brute_force_bitmap():
    rng = random.Random(4)
    slab = 256
    for _ in range(50):
        pool = Pool(8 * slab, slab)
        segs = [8]
        live = {}
        for _ in range(200):
            op = rng.random()
            try:
                if op < 0.45:
                    n = rng.randint(1, 5 * slab)
                    live[pool.alloc(n)] = n
                elif op < 0.75 and live:
                    off = rng.choice(list(live))
                    pool.free(off)
                    del live[off]
                elif op < 0.85:
                    k = rng.randint(1, 6)
                    pool.grow(k * slab)
                    segs.append(k)
                else:
                    first = sum(segs[:-1]) * slab
                    busy = any(off + -(-n // slab) * slab > first for off, n in live.items())
                    if len(segs) == 1:
                        with pytest.raises(OracleError) as ei:
                            pool.shrink()
                        assert ei.value.code == EINVAL
                    elif busy:
                        with pytest.raises(OracleError) as ei:
                            pool.shrink()
                        assert ei.value.code == EBUSY
                    else:
                        assert pool.shrink() == segs.pop() * slab
            except OracleError as e:
                assert e.code == -2
            assert pool.total_bytes == sum(segs) * slab
            assert pool.live_bytes == sum(-(-n // slab) * slab for n in live.values())


# ---- the library's host code against the oracle -------------------------------------------------

def test_library_sizer_and_planner_match_oracle():
    from paper_2411_01830_amd import binding as ft
    rng = random.Random(31)
    for _ in range(40):
        q = rng.choice([0.0, 0.5, 0.9, 0.99])
        floor = rng.randint(0, 5000)
        lib, orc = ft.Sizer(floor, q, 30.0), Sizer(floor, q or 0.99, 30.0)
        t = 0.0
        for _ in range(150):
            t += rng.choice([0.001, 0.5, 2.0, 40.0]) * rng.random()
            f = rng.randint(0, 3)
            size, con = rng.randint(0, 1 << 30), rng.randint(1, 9)
            lib.observe(f, t, size, con)
            orc.observe(f, t, size, con)
            for dt in (0.0, 0.3, 5.0, 31.0, 100.0):
                assert lib.target(t + dt) == orc.target(t + dt)
        lib.close()
    for _ in range(500):
        n = rng.randint(0, 14)
        objs = [dict(id=rng.randint(0, 1 << 40) * 16 + i, bytes=rng.randint(1, 1 << 20), queue_pos=rng.randint(0, 5),
                     resident=rng.random() < 0.6) for i in range(n)]
        cap, inc = rng.randint(0, 6 << 20), rng.randint(0, 1 << 20)
        assert ft.migrate_plan(objs, cap, inc, ft.FT_EVICT_QUEUE_AWARE) == plan_queue_aware(objs, cap, inc)
        assert ft.migrate_plan(objs, cap, inc, ft.FT_EVICT_LRU) == plan_lru(objs, cap, inc)


def test_library_pool_shrink_matches_oracle():
    from paper_2411_01830_amd import binding as ft
    rng = random.Random(6)
    slab = 4096
    base = 0x7000000000
    pool = ft.pool_create(base, 16 * slab, slab, 0)
    orc = Pool(16 * slab, slab)
    seg_bases = [base]
    live = []
    for step in range(600):
        op = rng.random()
        if op < 0.45:
            n = rng.randint(1, 9 * slab)
            try:
                want = orc.alloc(n)
            except OracleError as e:
                with pytest.raises(ft.FtError) as ei:
                    ft.slab_alloc(pool, n)
                assert ei.value.code == e.code
                continue
            assert ft.slab_alloc(pool, n) == want
            live.append(want)
        elif op < 0.75 and live:
            off = live.pop(rng.randrange(len(live)))
            orc.free(off)
            ft.slab_free(pool, off)
        elif op < 0.85:
            k = rng.randint(1, 8) * slab
            seg_bases.append(seg_bases[-1] + (1 << 30))
            orc.grow(k)
            ft.pool_grow(pool, seg_bases[-1], k)
        else:
            try:
                want = orc.shrink()
            except OracleError as e:
                with pytest.raises(ft.FtError) as ei:
                    ft.pool_shrink(pool)
                assert ei.value.code == e.code
                continue
            assert ft.pool_shrink(pool) == (seg_bases.pop(), want)
        assert ft.pool_usage(pool) == (orc.total_bytes, orc.live_bytes)
    ft.pool_destroy(pool)


def _oracle_store(capacity, pool_bytes=1 << 20, spill_bytes=1 << 20, slab=4096):
    from oracle import OracleEngine
    from oracle.store import Store
    from workloads import make_descs, FT_HOST, FT_POOL
    eng = OracleEngine()
    eng.host_arena(spill_bytes + 4096)
    eng.pool_create(pool_bytes, slab)
    return eng, Store(eng, 4096, spill_bytes, capacity, 4096, make_descs, FT_HOST, FT_POOL)


def test_store_follows_the_papers_example():
    """Sec. 7.2's example as a run of the store: the outputs of a1 and a2 fill it, b1 is next in the
    queue and b2 after it. A third output arrives: the output whose consumer is furthest back (a2's)
    goes to the host, not the oldest one (a1's, which b1 is about to read); once b1 is done with a1's
    output, a2's comes back before b2 asks for it, so b2 does not stall."""
    eng, st = _oracle_store(capacity=2 * 8192)
    o1 = st.put(1, 8192, 0)
    o2 = st.put(2, 8192, 1)
    eng.write_pool(o1, np.full(8192, 11, np.uint8))
    eng.write_pool(o2, np.full(8192, 22, np.uint8))
    o3 = st.put(3, 8192, 2)
    eng.write_pool(o3, np.full(8192, 33, np.uint8))
    # a3's own consumer is the furthest of all, but the rule only moves what is already stored: a2's goes
    assert [e for e in st.log if e[0] == "out"] == [("out", 2)]
    assert st.get(1) == (o1, False)
    st.done(1)
    assert ("in", 2, st.objs[2]["off"]) in st.log            # came back as soon as there was room
    st.advance(1)
    off, was_out = st.get(2)
    assert not was_out and st.stalls == 0
    assert np.all(eng.read_pool(off, 8192) == 22)            # and its bytes made the round trip


def test_store_random_runs_keep_the_budget_and_the_bytes():
    """Random puts, gets, dones and queue steps: the pool never holds more than the budget, a result
    read after any number of moves is the bytes that were stored, a get of a resident result moves
    nothing, no eviction is made that the budget did not require, spilled copies never overlap."""
    rng = np.random.default_rng(5)
    for trial in range(20):
        cap = int(rng.integers(6, 20)) * 4096
        eng, st = _oracle_store(capacity=cap)
        content = {}
        next_id = 0
        for step in range(120):
            op = rng.choice(["put", "put", "get", "done", "advance"])
            ids = sorted(st.objs)
            if op == "put":
                n = int(rng.integers(1, 5 * 4096))
                before_out = sum(1 for e in st.log if e[0] == "out")
                res_before = st.resident_bytes()
                off = st.put(next_id, n, int(rng.integers(0, 12)))
                data = rng.integers(0, 256, n, dtype=np.uint8)
                eng.write_pool(off, data)
                content[next_id] = data
                outs = [e[1] for e in st.log if e[0] == "out"][before_out:]
                if outs:        # without the last eviction the budget would have been passed
                    assert res_before - sum(len(content[i]) for i in outs[:-1]) + n > cap
                next_id += 1
            elif op == "get" and ids:
                i = int(rng.choice(ids))
                moves = len(st.log)
                resident = st.objs[i]["resident"]
                off, was_out = st.get(i)
                assert was_out == (not resident)
                if resident:
                    assert len(st.log) == moves
                assert np.array_equal(eng.read_pool(off, len(content[i])), content[i])
            elif op == "done" and ids:
                i = int(rng.choice(ids))
                st.get(i)
                st.done(i)
                del content[i]
            elif op == "advance":
                st.advance(int(rng.integers(0, 3)))
            assert st.resident_bytes() <= cap
            spans = sorted((o["spill"], o["spill"] + o["bytes"]) for o in st.objs.values() if not o["resident"])
            assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))
        for i in sorted(st.objs):
            off, _ = st.get(i)
            assert np.array_equal(eng.read_pool(off, len(content[i])), content[i])
