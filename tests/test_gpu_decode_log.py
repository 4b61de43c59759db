"""What the copy kernel's own ticket decode produced (the FT_LOG record it writes itself), ticket by
ticket, against the oracle's proportional chunk order of Sec. 6.1 cut into tiles.

The byte images of the other tests prove that the tickets of a launch cover every byte once; they do
not prove the ORDER the kernel follows. Here every ticket's (function, chunk, stream offset, bytes) as
decoded on the device by the hot path itself is compared with oracle.stride_order: all five workloads,
the routes on which a small job travels with its launch (including the one-descriptor shortcut), jobs
with a descriptor-table entry per tile, and open jobs whose later orders start in the middle of the
streams."""
import time

import numpy as np
import pytest

from oracle import OracleEngine
from oracle.batches import batched_order
from oracle.schedule import chunk_count
from workloads import configs, runner, make_descs, FT_HOST, FT_POOL
from workloads import format as fmt

pytestmark = pytest.mark.gpu
KiB, MiB = 1 << 10, 1 << 20


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2411_01830_amd import binding, harness
    assert torch.cuda.is_available()
    return binding, harness


def _class_of(d):
    return 2 if (d["src_space"] == FT_POOL and d["dst_space"] == FT_POOL) else (0 if d["dst_space"] == FT_POOL else 1)


def _stream_bytes(descs, nfunc, cls):
    S = [0] * nfunc
    for d in descs:
        if _class_of(d) == cls:
            S[int(d["func"])] += int(d["row_bytes"]) * int(d["rows"])
    return S


def _tiles(order, S, C, tile):
    """The oracle's chunk order with every chunk cut into tiles of `tile` bytes, in ascending order."""
    out = []
    for f, k in order:
        lo, hi = k * C, min((k + 1) * C, S[f])
        b = lo
        while b < hi:
            out.append((f, k, b, min(tile, lo + C - b, hi - b)))
            b += tile
    return out


def _log_tuples(log):
    return list(zip(log["func"].tolist(), log["chunk"].tolist(), log["byte_off"].tolist(), log["bytes"].tolist()))


def _check_job(binding, eng, orc, job_g, job_o, descs, nfunc, C, classes=(0, 1, 2)):
    st = binding.job_stats(eng.pool, job_g)
    seen = 0
    for cls in classes:
        order = orc.job_schedule(job_o, cls)
        if not order:
            continue
        S = _stream_bytes(descs, nfunc, cls)
        want = _tiles(order, S, C, st.cls[cls].tile_bytes)
        got = _log_tuples(binding.job_log(eng.pool, job_g, cls))
        assert len(got) == st.cls[cls].tickets == len(want), (cls, len(got), len(want))
        if got != want:
            bad = next(i for i, (a, b) in enumerate(zip(got, want)) if a != b)
            raise AssertionError(f"class {cls}: ticket {bad} decoded as {got[bad]}, the oracle's order gives {want[bad]}")
        seen += len(got)
    return st, seen


SCALED = [("tiny", 0.3), ("traffic", 0.2), ("feature", 0.02), ("contended", 0.01), ("large_mixed", 0.008)]


@pytest.mark.parametrize("name,scale", SCALED)
def test_device_decode_follows_the_oracle_order(gpu, name, scale):
    binding, harness = gpu
    print(f"case device decode {name} scale {scale}", flush=True)
    plan = configs.CONFIGS[name](scale)
    orc = OracleEngine()
    rec_o = runner.run_plan(plan, orc)
    eng = harness.GpuEngine()
    try:
        rec_g = runner.run_plan(plan, eng, flags=fmt.FT_VALIDATE | fmt.FT_LOG)
        total = 0
        for jname, job in rec_g.jobs.items():
            _, n = _check_job(binding, eng, orc, job, rec_o.jobs[jname], rec_g.descs[jname], len(rec_g.weights[jname]),
                              rec_g.chunk_bytes[jname])
            total += n
            binding.job_release(eng.pool, job)
        assert total > 0
    finally:
        eng.close()


def _pair(gpu, host, pool, slab, seed):
    _, harness = gpu
    orc, eng = OracleEngine(), harness.GpuEngine()
    rng = np.random.default_rng(seed)
    data = rng.integers(0, 256, host // 2, dtype=np.uint8)
    for e in (orc, eng):
        e.host_arena(host)
        e.pool_create(pool, slab)
        e.write_host(0, data)
    return orc, eng, rng


def _alloc(orc, eng, n, rng=None):
    a = orc.slab_alloc(n)
    assert eng.slab_alloc(n) == a
    if rng is not None:
        fill = rng.integers(0, 256, n, dtype=np.uint8)
        orc.write_pool(a, fill)
        eng.write_pool(a, fill)
    return a


def _images_equal(orc, eng):
    import torch
    assert np.array_equal(eng.host_np[:len(orc.host_mem)], orc.host_mem), "host image differs"
    assert np.array_equal(torch.cat([t for t, _ in eng.segments]).cpu().numpy(), orc.pool_mem), "pool image differs"


def test_jobs_that_travel_with_their_launch(gpu):
    """One function with one descriptor (the decode's shortcut that reads no schedule table), and small
    jobs of several functions, in every link class: a tile per workgroup, and more tiles than workgroups
    (a counter pair of the device)."""
    binding, _ = gpu
    orc, eng, rng = _pair(gpu, 64 * MiB, 160 * MiB, 64 * KiB, 31)
    try:
        C = 256 * KiB
        host_dst = [32 * MiB]

        def rec(f, cls, n):
            if cls == 0:
                return dict(func=f, src_space=FT_HOST, dst_space=FT_POOL, src=16 * int(rng.integers(0, 1000)) + 3,
                            dst=_alloc(orc, eng, n + 32) + 5, row_bytes=n)
            if cls == 1:
                at = host_dst[0]
                host_dst[0] += (n + 63) // 16 * 16
                return dict(func=f, src_space=FT_POOL, dst_space=FT_HOST, src=_alloc(orc, eng, n + 32, rng) + 7, dst=at + 1,
                            row_bytes=n)
            return dict(func=f, src_space=FT_POOL, dst_space=FT_POOL, src=_alloc(orc, eng, n + 32, rng) + 16,
                        dst=_alloc(orc, eng, n + 32) + 16, row_bytes=n)
        cases = []
        for cls in (0, 1, 2):
            cases.append((cls, [rec(0, cls, 3 * MiB + 12345)], [1]))                       # single, a tile per workgroup
            cases.append((cls, [rec(0, cls, (20 if cls == 2 else 3) * MiB + 17)], [5]))     # single, pool->pool needs a counter
            cases.append((cls, [rec(f, cls, n) for f, n in enumerate((700 * KiB + 3, 64, 2 * MiB, 300 * KiB))],
                          [1, 3, 2, 2]))
        in_launch = 0
        for cls, recs, w in cases:
            d = make_descs(recs)
            print(f"case in-launch class {cls} descriptors {len(recs)}", flush=True)
            jo = orc.submit(d, w, C)
            orc.wait(jo)
            jg = eng.submit(d, w, C, fmt.FT_LOG | fmt.FT_VALIDATE)
            eng.wait(jg)
            st, _ = _check_job(binding, eng, orc, jg, jo, d, len(w), C, classes=(cls,))
            in_launch += st.cls[cls].in_launch
            binding.job_release(eng.pool, jg)
        assert in_launch == len(cases)          # every one of them went with its launch
        _images_equal(orc, eng)
    finally:
        eng.close()


def test_descriptor_table_per_tile(gpu):
    """Many descriptors per chunk: the planner lists a descriptor per tile and the decode takes the tile's
    first descriptor from there (no search). Rows gathered from a pitched source and short contiguous pieces."""
    binding, _ = gpu
    orc, eng, rng = _pair(gpu, 1 * MiB, 96 * MiB, 16 * KiB, 32)
    try:
        C = 256 * KiB
        recs = []
        for i in range(420):
            f = i % 3
            if i % 2:
                rb, rows = int(rng.integers(20, 200)), int(rng.integers(2, 90))
                pitch = rb + int(rng.integers(0, 300))
                recs.append(dict(func=f, src_space=FT_POOL, dst_space=FT_POOL, src=_alloc(orc, eng, rows * pitch + 32, rng) + int(rng.integers(0, 16)),
                                 dst=_alloc(orc, eng, rows * rb + 32) + int(rng.integers(0, 16)), row_bytes=rb, rows=rows,
                                 src_pitch=pitch, dst_pitch=rb))
            else:
                n = int(rng.integers(1, 30000))
                recs.append(dict(func=f, src_space=FT_POOL, dst_space=FT_POOL, src=_alloc(orc, eng, n + 32, rng) + int(rng.integers(0, 16)),
                                 dst=_alloc(orc, eng, n + 32) + int(rng.integers(0, 16)), row_bytes=n))
        d = make_descs(recs)
        w = [2, 1, 5]
        jo = orc.submit(d, w, C)
        orc.wait(jo)
        jg = eng.submit(d, w, C, fmt.FT_LOG | fmt.FT_VALIDATE)
        eng.wait(jg)
        st, n = _check_job(binding, eng, orc, jg, jo, d, 3, C, classes=(2,))
        assert n > 3 * 4 and st.cls[2].in_launch == 0
        binding.job_release(eng.pool, jg)
        _images_equal(orc, eng)
    finally:
        eng.close()


def _h2p_job(orc, eng, rng, sizes, host_limit):
    recs = []
    for f, n in enumerate(sizes):
        a = _alloc(orc, eng, n + 32)
        src = int(rng.integers(0, (host_limit - n) // 16)) * 16 + int(rng.integers(0, 2)) * 3
        recs.append(dict(func=f, src_space=FT_HOST, dst_space=FT_POOL, src=src, dst=a + int(rng.integers(0, 16)), row_bytes=n))
    return recs


@pytest.mark.parametrize("batch,depth", [(5, 2), (3, 1)])
def test_open_sequence_decodes_the_batched_order(gpu, batch, depth):
    """An open job, two jobs merged while it runs and a change of weights: every later order starts in the
    middle of the streams (chunks already triggered) and every batch in the middle of an order's tickets.
    The kernel's per-ticket record must be the oracle's batches, given the batch numbers at which the
    library says the jobs joined and the weights changed, cut into tiles; and the progress counters end at
    the stream sizes."""
    binding, _ = gpu
    orc, eng, rng = _pair(gpu, 192 * MiB, 256 * MiB, 64 * KiB, 40 + batch)
    try:
        C = 256 * KiB
        binding.set_batch(eng.pool, batch, depth)
        jobs_sizes = [[36 * MiB + 100, 24 * MiB + 48, 17 * MiB + 5], [1 * MiB + 7, 300 * KiB], [3 * MiB, 2 * MiB + 1, 64 * KiB]]
        jobs_w = [[1, 2, 1], [8, 8], [4, 1, 2]]
        new_w0 = [3, 1, 1]
        descs = [make_descs(_h2p_job(orc, eng, rng, s, 96 * MiB)) for s in jobs_sizes]
        for d, w in zip(descs, jobs_w):
            orc.wait(orc.submit(d, w, C))
        print(f"case open sequence with device log batch={batch} depth={depth}", flush=True)
        handles = [eng.submit(descs[0], jobs_w[0], C, fmt.FT_OPEN | fmt.FT_KEEP | fmt.FT_LOG)]
        merged = {}
        for i in (1, 2):
            try:
                handles.append(eng.merge(handles[0], descs[i], jobs_w[i], fmt.FT_KEEP))
                merged[i] = True
            except binding.FtError as e:
                assert e.code == fmt.FT_ECLOSED
                handles.append(eng.submit(descs[i], jobs_w[i], C, fmt.FT_KEEP))
            time.sleep(0.0002)
        rw_at = binding.job_reweight(eng.pool, handles[0], new_w0)[0]
        mid, _ = binding.job_progress(eng.pool, handles[0], 0, 3)
        for h in reversed(handles):
            eng.wait(h)
        _images_equal(orc, eng)
        done, nb = binding.job_progress(eng.pool, handles[0], 0, 3)
        assert done == jobs_sizes[0] and all(m <= s for m, s in zip(mid, jobs_sizes[0]))
        spec = [{"n": [chunk_count(s, C) for s in jobs_sizes[0]], "w": jobs_w[0]}]
        if rw_at is not None:
            spec[0]["reweight"] = [(rw_at, new_w0)]
        index = {handles[0]: 0}
        sizes_of = {0: jobs_sizes[0]}
        for i in (1, 2):
            if i not in merged:
                continue
            index[handles[i]] = len(spec)
            sizes_of[len(spec)] = jobs_sizes[i]
            spec.append({"n": [chunk_count(s, C) for s in jobs_sizes[i]], "w": jobs_w[i],
                         "arrive": binding.job_arrival(eng.pool, handles[i], 0)})
            assert binding.job_progress(eng.pool, handles[i], 0, len(jobs_sizes[i]))[0] == jobs_sizes[i]
        want_batches = batched_order(spec, batch)
        assert nb == len(want_batches)
        st = binding.job_stats(eng.pool, handles[0])
        tile = st.cls[0].tile_bytes
        want = []
        for b, chunks in enumerate(want_batches):
            for j, f, k in chunks:
                S = sizes_of[j][f]
                lo, hi = k * C, min((k + 1) * C, S)
                at = lo
                while at < hi:
                    want.append((j, f, k, at, min(tile, lo + C - at, hi - at), b))
                    at += tile
        log = binding.job_log(eng.pool, handles[0], 0)
        who = binding.job_log_jobs(eng.pool, handles[0], 0)
        got = [(index[j], f, k, o, n, b) for j, (f, k, o, n), b in
               zip(who["job"].tolist(), _log_tuples(log), who["batch"].tolist())]
        assert len(got) == len(want)
        if got != want:
            bad = next(i for i, (a, b) in enumerate(zip(got, want)) if a != b)
            raise AssertionError(f"ticket {bad} of the sequence decoded as {got[bad]}, the oracle gives {want[bad]}")
        assert np.all(log["t_end_ns"] >= log["t_begin_ns"])
        print("arrivals", [s.get("arrive", 0) for s in spec], "reweight at", rw_at, "batches", nb, "tickets", len(got), flush=True)
        for h in handles:
            binding.job_release(eng.pool, h)
    finally:
        eng.close()
