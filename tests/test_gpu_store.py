"""Elastic data store (Sec. 7) end to end on the GPU: the pool grows and shrinks with the
histogram rule, data is moved to host memory and back by the queue-aware rule, every move is
an ordinary transfer of the engine. The oracle runs the same scenario with its own policies;
decisions, allocation offsets and every byte must agree."""
import numpy as np
import pytest

from oracle import OracleEngine
from oracle.store import Sizer as OracleSizer, plan_queue_aware
from workloads import make_descs, FT_HOST, FT_POOL

pytestmark = pytest.mark.gpu

KiB, MiB = 1 << 10, 1 << 20


def _run_store(eng, sizer, planner, usage, shrink, sizes, lookahead, capacity, seg, results_off, spill_off, chunk):
    """Two-stage workflow under memory pressure. Returns the log of decisions."""
    log = []
    objs = {}          # id -> dict(bytes, resident, off (pool) or spill (host offset))
    spill_next = [spill_off]
    nseg = [1]
    n = len(sizes)

    def view(head, skip=None):
        return [dict(id=i, bytes=o["bytes"], queue_pos=i - head, resident=o["resident"])
                for i, o in sorted(objs.items()) if i != skip]

    def move_out(i):
        o = objs[i]
        o["spill"] = spill_next[0]
        spill_next[0] += (o["bytes"] + 255) // 256 * 256
        d = make_descs([dict(func=0, src_space=FT_POOL, dst_space=FT_HOST, src=o["off"] + o["shift"], dst=o["spill"],
                             row_bytes=o["bytes"])])
        eng.wait(eng.submit(d, [1], chunk))
        eng.slab_free(o["off"])
        o["resident"] = False
        log.append(("out", i))

    def alloc(nbytes, t):
        # the pool follows the histogram rule's target, in whole segments, never below what is live
        total, live = usage()
        want = max(sizer.target(t), live + nbytes)
        while total < want:
            eng.pool_grow(seg)
            nseg[0] += 1
            total += seg
            log.append(("grow", nseg[0]))
        return eng.slab_alloc(nbytes)

    def move_in(i, t):
        o = objs[i]
        o["off"] = alloc(o["bytes"] + 16, t)
        d = make_descs([dict(func=0, src_space=FT_HOST, dst_space=FT_POOL, src=o["spill"], dst=o["off"] + o["shift"],
                             row_bytes=o["bytes"])])
        eng.wait(eng.submit(d, [1], chunk))
        o["resident"] = True
        log.append(("in", i, o["off"]))

    def store(i, t):
        ev, _ = planner(view(max(i - lookahead, 0)), capacity, sizes[i])
        for e in ev:
            move_out(e)
        shift = i % 16
        off = alloc(sizes[i] + 16, t)
        d = make_descs([dict(func=0, src_space=FT_HOST, dst_space=FT_POOL, src=4096 + i * 1777, dst=off + shift,
                             row_bytes=sizes[i])])
        eng.wait(eng.submit(d, [1], chunk))
        objs[i] = dict(bytes=sizes[i], resident=True, off=off, shift=shift)
        sizer.observe(0, t, sizes[i], min(lookahead, n - 1) + 1)
        log.append(("store", i, off))

    for i in range(min(lookahead, n)):
        store(i, float(i))
    for head in range(n):
        t = float(head + lookahead)
        if head + lookahead < n:
            store(head + lookahead, t)
        if not objs[head]["resident"]:
            ev, _ = planner(view(head, skip=head), capacity, sizes[head])
            for e in ev:
                move_out(e)
            move_in(head, t)
            log.append(("stall", head))
        o = objs.pop(head)
        # the consumer: copy the first 4 KiB of its input to its slot in the results area
        take = min(4096, o["bytes"])
        d = make_descs([dict(func=0, src_space=FT_POOL, dst_space=FT_HOST, src=o["off"] + o["shift"],
                             dst=results_off + head * 4096, row_bytes=take)])
        eng.wait(eng.submit(d, [1], chunk))
        eng.slab_free(o["off"])
        ev, rl = planner(view(head + 1), capacity, 0)
        for e in ev:
            move_out(e)
        for r in rl:
            move_in(r, t)
        # give memory back while the target allows it and the tail of the pool is empty
        while nseg[0] > 1:
            total, live = usage()
            if total - seg < max(sizer.target(t), live):
                break
            try:
                shrink()
            except Exception as e:      # noqa: BLE001
                assert getattr(e, "code", None) == -5
                break
            nseg[0] -= 1
            log.append(("shrink", nseg[0]))
    return log


def test_elastic_store_matches_oracle():
    import torch
    from paper_2411_01830_amd import binding as ft, harness
    rng = np.random.default_rng(3)
    n, lookahead = 48, 6
    sizes = [int(x) for x in rng.integers(200 * KiB, 1500 * KiB, n)]
    sizes[20:28] = [int(x) for x in rng.integers(2 * MiB, 3 * MiB, 8)]     # a burst of large results
    capacity, seg = 8 * MiB, 4 * MiB
    host_bytes = 96 * MiB
    results_off, spill_off = 1 * MiB, 8 * MiB
    data = rng.integers(0, 256, 1 * MiB, dtype=np.uint8)

    orc = OracleEngine()
    orc.host_arena(host_bytes)
    orc.pool_create(seg, 64 * KiB)
    orc.write_host(0, data)
    osz = OracleSizer(seg, 0.99, 3.0)
    log_o = _run_store(orc, osz, plan_queue_aware, lambda: (orc.pool.total_bytes, orc.pool.live_bytes),
                       orc.pool_shrink, sizes, lookahead, capacity, seg, results_off, spill_off, 256 * KiB)

    eng = harness.GpuEngine()
    try:
        eng.host_arena(host_bytes)
        eng.pool_create(seg, 64 * KiB)
        eng.write_host(0, data)
        gsz = ft.Sizer(seg, 0.99, 3.0)

        def gpu_shrink():
            base, nbytes = ft.pool_shrink(eng.pool)
            t, first = eng.segments.pop()
            assert t.data_ptr() == base and t.numel() == nbytes
            eng.total -= nbytes

        log_g = _run_store(eng, gsz, lambda o, c, i: ft.migrate_plan(o, c, i), lambda: ft.pool_usage(eng.pool),
                           gpu_shrink, sizes, lookahead, capacity, seg, results_off, spill_off, 256 * KiB)
        assert log_g == log_o
        kinds = {k[0] for k in log_g}
        assert {"store", "out", "in", "grow", "shrink"} <= kinds, kinds      # the scenario exercises every move
        assert np.array_equal(eng.host_np, orc.host_mem), "host image (results and spill area) differs"
        got = torch.cat([t for t, _ in eng.segments]).cpu().numpy()
        assert np.array_equal(got, orc.pool_mem), "pool image differs"
        # every consumer saw the bytes its producer stored
        for i in range(n):
            take = min(4096, sizes[i])
            src = 4096 + i * 1777
            assert np.array_equal(eng.host_np[results_off + i * 4096:results_off + i * 4096 + take],
                                  orc.host_mem[src:src + take])
        print("moves:", {k: sum(1 for x in log_g if x[0] == k) for k in sorted(kinds)}, flush=True)
        gsz.close()
    finally:
        eng.close()


def test_native_store_matches_the_oracle_store():
    """The library's own store (ft_store_*) against the oracle's store on a two-stage workflow under
    memory pressure with out-of-order consumers: every offset it hands out, every stall, the counts and
    bytes of its moves, and afterwards the whole pool, the whole spill arena and what each consumer read."""
    import torch
    from oracle.store import Store as OracleStore
    from paper_2411_01830_amd import binding as ft, harness
    rng = np.random.default_rng(11)
    n, lookahead = 60, 7
    sizes = [int(x) for x in rng.integers(100 * KiB, 900 * KiB, n)]
    sizes[25:31] = [int(x) for x in rng.integers(1500 * KiB, 2500 * KiB, 6)]
    capacity, pool_bytes = 5 * MiB, 12 * MiB
    spill_off, spill_bytes, results_off = 4 * MiB, 40 * MiB, 1 * MiB
    payload = [rng.integers(0, 256, s, dtype=np.uint8) for s in sizes]
    order = list(range(n))
    for k in range(0, n - 3, 5):                      # now and then a later request overtakes
        order[k + 1], order[k + 2] = order[k + 2], order[k + 1]

    def run(eng, store, after_put=None):
        trace = []
        stored = 0
        for step, head in enumerate(order):
            while stored < n and stored <= step + lookahead:
                off = store.put(stored, sizes[stored], stored - step if stored > step else 0)
                if after_put is not None:
                    after_put()
                eng.write_pool(off, payload[stored])
                trace.append(("put", stored, off))
                stored += 1
            off, was_out = store.get(head)
            trace.append(("get", head, off, was_out))
            take = min(4096, sizes[head])
            d = make_descs([dict(func=0, src_space=FT_POOL, dst_space=FT_HOST, src=off, dst=results_off + head * 4096,
                                 row_bytes=take)])
            eng.wait(eng.submit(d, [1], 256 * KiB))
            store.done(head)
            store.advance(1)
        return trace

    orc = OracleEngine()
    orc.host_arena(spill_off + spill_bytes)
    orc.pool_create(pool_bytes, 64 * KiB)
    ost = OracleStore(orc, spill_off, spill_bytes, capacity, 256 * KiB, make_descs, FT_HOST, FT_POOL)
    trace_o = run(orc, ost)

    eng = harness.GpuEngine()
    try:
        eng.host_arena(spill_off + spill_bytes)
        eng.pool_create(pool_bytes, 64 * KiB)
        gst = ft.Store(eng.pool, eng.host.data_ptr() + spill_off, spill_bytes, capacity, 256 * KiB,
                       torch.cuda.current_stream().cuda_stream)
        in_flight = []
        trace_g = run(eng, gst, lambda: in_flight.append(gst.stats().moves_in_flight))
        assert trace_g == trace_o
        # moves are not waited for by the calls that start them: some were still unsettled when a call returned
        assert max(in_flight) >= 1, in_flight
        gst.sync()                      # quiescent point: memory now holds what the decisions imply
        st = gst.stats()
        assert st.moves_in_flight == 0
        outs = [e for e in ost.log if e[0] == "out"]
        ins = [e for e in ost.log if e[0] == "in"]
        assert (st.moved_out, st.moved_in, st.stalls) == (len(outs), len(ins), ost.stalls)
        assert st.bytes_out == sum(sizes[e[1]] for e in outs) and st.bytes_in == sum(sizes[e[1]] for e in ins)
        assert st.objects == 0 and st.resident_bytes == 0
        assert len(outs) >= 10 and ost.stalls >= 1 and len(ins) > ost.stalls      # moves, stalls and early returns all occur
        assert np.array_equal(eng.host_np, orc.host_mem), "host image (results and spill arena) differs"
        got = torch.cat([t for t, _ in eng.segments]).cpu().numpy()
        assert np.array_equal(got, orc.pool_mem), "pool image differs"
        for i in range(n):
            take = min(4096, sizes[i])
            assert np.array_equal(eng.host_np[results_off + i * 4096:results_off + i * 4096 + take], payload[i][:take]), i
        print("store moves:", {"out": st.moved_out, "in": st.moved_in, "stalls": st.stalls}, flush=True)
        gst.close()
    finally:
        eng.close()
