"""Open jobs (batched transfer triggering, Sec. 6.1) against the oracle: bytes, and the
order of the batches given the batch at which the library says each job joined."""
import time

import numpy as np
import pytest

from oracle import OracleEngine
from oracle.batches import batched_order
from oracle.schedule import chunk_count
from workloads import make_descs, FT_HOST, FT_POOL
from workloads import format as fmt

pytestmark = pytest.mark.gpu

KiB, MiB = 1 << 10, 1 << 20


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2411_01830_amd import binding, harness
    assert torch.cuda.is_available()
    return binding, harness


def _engines(gpu, host_bytes, pool_bytes, slab=64 * KiB, seed=0):
    _, harness = gpu
    orc, eng = OracleEngine(), harness.GpuEngine()
    rng = np.random.default_rng(seed)
    data = rng.integers(0, 256, host_bytes // 2, dtype=np.uint8)
    for e in (orc, eng):
        e.host_arena(host_bytes)
        e.pool_create(pool_bytes, slab)
        e.write_host(0, data)
    return orc, eng, rng


def _images_equal(orc, eng):
    import torch
    assert np.array_equal(eng.host_np[:len(orc.host_mem)], orc.host_mem), "host image differs"
    got = torch.cat([t for t, _ in eng.segments]).cpu().numpy()
    assert np.array_equal(got, orc.pool_mem), "pool image differs"


def _h2p_job(orc, eng, rng, sizes, host_limit):
    """One host->pool descriptor per function; returns (records, chunk streams)."""
    recs = []
    for f, n in enumerate(sizes):
        a = orc.slab_alloc(n + 32)
        assert eng.slab_alloc(n + 32) == a
        src = int(rng.integers(0, (host_limit - n) // 16)) * 16 + int(rng.integers(0, 2)) * 3
        recs.append(dict(func=f, src_space=FT_HOST, dst_space=FT_POOL, src=src, dst=a + int(rng.integers(0, 16)),
                         row_bytes=n))
    return recs


def test_open_job_alone_is_the_plain_order_in_batches(gpu):
    binding, _ = gpu
    orc, eng, rng = _engines(gpu, 64 * MiB, 96 * MiB)
    try:
        C = 256 * KiB
        sizes = [5 * MiB + 1234, 9 * MiB, 3 * MiB + 16, 700 * KiB]
        w = [1, 2, 4, 1]
        recs = _h2p_job(orc, eng, rng, sizes, 32 * MiB)
        d = make_descs(recs)
        binding.set_batch(eng.pool, 5, 2)
        orc.wait(orc.submit(d, w, C))
        job = eng.submit(d, w, C, fmt.FT_OPEN | fmt.FT_KEEP | fmt.FT_VALIDATE)
        assert binding.job_arrival(eng.pool, job, 0) == 0
        eng.wait(job)
        _images_equal(orc, eng)
        got = binding.job_batches(eng.pool, job, 0)
        n = [chunk_count(s, C) for s in sizes]
        want = batched_order([{"n": n, "w": w}], 5)
        assert [[(f, k) for _, f, k in b] for b in got] == [[(f, k) for _, f, k in b] for b in want]
        assert all(j == job for b in got for j, _, _ in b)
        st = binding.job_stats(eng.pool, job)
        assert st.cls[0].payload_bytes == sum(sizes) and st.cls[0].chunks == sum(n)
        binding.job_release(eng.pool, job)
    finally:
        eng.close()


@pytest.mark.parametrize("batch,depth", [(5, 2), (2, 1), (16, 3)])
def test_merged_jobs_match_oracle(gpu, batch, depth):
    """A long host->pool job, then two more merged while it runs. Whatever batch each one
    joins at (the library says), the batches must be the oracle's for those arrivals and the
    bytes the plain copy."""
    binding, _ = gpu
    orc, eng, rng = _engines(gpu, 192 * MiB, 256 * MiB, seed=batch)
    try:
        C = 256 * KiB
        binding.set_batch(eng.pool, batch, depth)
        jobs_sizes = [[40 * MiB, 24 * MiB + 48, 17 * MiB + 5], [1 * MiB + 7, 300 * KiB], [3 * MiB, 2 * MiB + 1, 64 * KiB]]
        jobs_w = [[1, 2, 1], [8, 8], [4, 1, 2]]
        descs = [make_descs(_h2p_job(orc, eng, rng, s, 96 * MiB)) for s in jobs_sizes]
        for d, w in zip(descs, jobs_w):
            orc.wait(orc.submit(d, w, C))
        print(f"open job batch={batch} depth={depth}", flush=True)
        handles = [eng.submit(descs[0], jobs_w[0], C, fmt.FT_OPEN | fmt.FT_KEEP)]
        closed = []
        for i in (1, 2):
            try:
                handles.append(eng.merge(handles[0], descs[i], jobs_w[i], fmt.FT_KEEP))
            except binding.FtError as e:          # the open job was already done: legal, run it alone
                assert e.code == fmt.FT_ECLOSED
                closed.append(i)
                handles.append(eng.submit(descs[i], jobs_w[i], C, fmt.FT_KEEP))
            time.sleep(0.0002)
        for h in reversed(handles):
            eng.wait(h)
        _images_equal(orc, eng)
        spec = [{"n": [chunk_count(s, C) for s in jobs_sizes[0]], "w": jobs_w[0]}]
        index = {handles[0]: 0}
        for i in (1, 2):
            if i in closed:
                continue
            a = binding.job_arrival(eng.pool, handles[i], 0)
            index[handles[i]] = len(spec)
            spec.append({"n": [chunk_count(s, C) for s in jobs_sizes[i]], "w": jobs_w[i], "arrive": a})
        got = binding.job_batches(eng.pool, handles[0], 0)
        got = [[(index[j], f, k) for j, f, k in b] for b in got]
        assert got == batched_order(spec, batch)
        print("arrivals", [s.get("arrive", 0) for s in spec], "batches", len(got), "closed", closed, flush=True)
        for h in handles:
            binding.job_release(eng.pool, h)
    finally:
        eng.close()


def test_merge_other_classes_and_busy_allocations(gpu):
    """pool->host and pool->pool traffic merged into an open job that has all three classes;
    allocations of a merged job stay busy until it has been waited for."""
    binding, _ = gpu
    orc, eng, rng = _engines(gpu, 128 * MiB, 256 * MiB, seed=5)
    try:
        C = 128 * KiB
        binding.set_batch(eng.pool, 4, 2)

        def alloc(n):
            a = orc.slab_alloc(n)
            assert eng.slab_alloc(n) == a
            return a

        def filled(n):
            a = alloc(n)
            data = rng.integers(0, 256, n, dtype=np.uint8)
            orc.write_pool(a, data)
            eng.write_pool(a, data)
            return a

        big = 24 * MiB
        recs0 = [dict(func=0, src_space=FT_HOST, dst_space=FT_POOL, src=4096, dst=alloc(big), row_bytes=big),
                 dict(func=1, src_space=FT_POOL, dst_space=FT_HOST, src=filled(big), dst=64 * MiB, row_bytes=big),
                 dict(func=2, src_space=FT_POOL, dst_space=FT_POOL, src=filled(big) + 3, dst=alloc(big) + 8,
                      row_bytes=big - 16)]
        small_src = filled(2 * MiB)
        small_dst = alloc(2 * MiB)
        recs1 = [dict(func=0, src_space=FT_POOL, dst_space=FT_HOST, src=small_src, dst=64 * MiB + big + 4096,
                      row_bytes=2 * MiB - 5),
                 dict(func=0, src_space=FT_HOST, dst_space=FT_POOL, src=20 * MiB + 1, dst=small_dst, row_bytes=1 * MiB)]
        d0, d1 = make_descs(recs0), make_descs(recs1)
        orc.wait(orc.submit(d0, [1, 1, 1], C))
        orc.wait(orc.submit(d1, [5], C))
        j0 = eng.submit(d0, [1, 1, 1], C, fmt.FT_OPEN | fmt.FT_KEEP)
        try:
            j1 = eng.merge(j0, d1, [5], fmt.FT_KEEP)
            merged = True
        except binding.FtError as e:
            assert e.code == fmt.FT_ECLOSED
            j1 = eng.submit(d1, [5], C, fmt.FT_KEEP)
            merged = False
        with pytest.raises(binding.FtError) as ei:
            eng.slab_free(small_dst)
        assert ei.value.code == fmt.FT_EBUSY
        eng.wait(j1)
        eng.slab_free(small_dst)
        orc.slab_free(small_dst)
        eng.wait(j0)
        _images_equal(orc, eng)
        print("merged" if merged else "closed before the merge", flush=True)
        # once everything is done the open job accepts nothing more
        with pytest.raises(binding.FtError) as ei:
            eng.merge(j0, d1[:1], [5])
        assert ei.value.code == fmt.FT_ECLOSED
        binding.job_release(eng.pool, j0)
        binding.job_release(eng.pool, j1)
    finally:
        eng.close()


def test_open_rejects_dma_and_keeps_its_log_until_dry(gpu):
    """The comparison path has no batches: FT_PATH_DMA with FT_OPEN is refused. FT_LOG is taken: the
    per-ticket record of the whole sequence is there once the class has run dry."""
    binding, _ = gpu
    orc, eng, rng = _engines(gpu, 4 * MiB, 8 * MiB)
    try:
        d = make_descs(_h2p_job(orc, eng, rng, [64 * KiB], 1 * MiB))
        with pytest.raises(binding.FtError) as ei:
            eng.submit(d, [1], 4096, fmt.FT_OPEN | fmt.FT_PATH_DMA)
        assert ei.value.code == fmt.FT_EINVAL
        orc.wait(orc.submit(d, [1], 4096))
        job = eng.submit(d, [1], 4096, fmt.FT_OPEN | fmt.FT_LOG)
        eng.wait(job)
        _images_equal(orc, eng)
        log = binding.job_log(eng.pool, job, 0)
        assert int(log["bytes"].sum()) == 64 * KiB and set(log["func"].tolist()) == {0}
        assert log["chunk"].tolist() == sorted(log["chunk"].tolist()) and int(log["chunk"].max()) == 15
        with pytest.raises(binding.FtError) as ei:          # the per-workgroup record is a closed job's
            binding.job_log_workgroups(eng.pool, job, 0, len(log["bytes"]))
        assert ei.value.code == fmt.FT_EINVAL
        binding.job_release(eng.pool, job)
    finally:
        eng.close()


@pytest.mark.parametrize("batch,depth,threads", [(5, 3, 4), (2, 1, 1), (3, 2, 2)])
def test_pageable_sources_through_the_ring(gpu, batch, depth, threads):
    """Sources in ordinary host memory (Sec. 6.1, circular pinned buffer): many more batches than
    ring slots, odd sizes and alignments, a pitched source, pinned and pageable descriptors mixed
    in one function, and a pageable job merged into a running one. Bytes must match the oracle."""
    from workloads import FT_PAGEABLE
    binding, _ = gpu
    orc, eng, rng = _engines(gpu, 64 * MiB, 192 * MiB, seed=17 + batch)
    try:
        C = 64 * KiB
        page = rng.integers(0, 256, 48 * MiB, dtype=np.uint8)
        for e in (orc, eng):
            e.pageable_arena(48 * MiB)
            e.write_pageable(0, page)
        binding.set_batch(eng.pool, batch, depth)
        binding.set_stage_threads(eng.pool, threads)

        def alloc(n):
            a = orc.slab_alloc(n)
            assert eng.slab_alloc(n) == a
            return a

        recs0 = [
            dict(func=0, src_space=FT_PAGEABLE, dst_space=FT_POOL, src=1, dst=alloc(9 * MiB) + 5, row_bytes=8 * MiB + 333),
            dict(func=1, src_space=FT_PAGEABLE, dst_space=FT_POOL, src=10 * MiB + 16, dst=alloc(3 * MiB), row_bytes=3 * MiB),
            # pinned and pageable pieces in one function's stream
            dict(func=1, src_space=FT_HOST, dst_space=FT_POOL, src=4096 + 3, dst=alloc(1 * MiB) + 1, row_bytes=700001),
            dict(func=1, src_space=FT_PAGEABLE, dst_space=FT_POOL, src=14 * MiB + 7, dst=alloc(1 * MiB), row_bytes=99),
            # rows of 200 bytes out of a pitch of 1000, packed at the destination
            dict(func=2, src_space=FT_PAGEABLE, dst_space=FT_POOL, src=16 * MiB + 9, dst=alloc(2 * MiB) + 2, row_bytes=200,
                 rows=9000, src_pitch=1000, dst_pitch=200),
            dict(func=2, src_space=FT_HOST, dst_space=FT_POOL, src=8 * MiB, dst=alloc(4 * MiB), row_bytes=4 * MiB),
        ]
        recs1 = [dict(func=0, src_space=FT_PAGEABLE, dst_space=FT_POOL, src=30 * MiB + 11, dst=alloc(2 * MiB) + 3,
                      row_bytes=1 * MiB + 17)]
        d0, d1 = make_descs(recs0), make_descs(recs1)
        orc.wait(orc.submit(d0, [1, 2, 3], C))
        orc.wait(orc.submit(d1, [9], C))
        print(f"pageable batch={batch} depth={depth} threads={threads}", flush=True)
        # the comparison path has no way for pageable memory
        with pytest.raises(binding.FtError) as ei:
            eng.submit(d1, [9], C, fmt.FT_PATH_DMA)
        assert ei.value.code == fmt.FT_EINVAL
        j0 = eng.submit(d0, [1, 2, 3], C, fmt.FT_OPEN | fmt.FT_KEEP | fmt.FT_VALIDATE)
        try:
            j1 = eng.merge(j0, d1, [9], fmt.FT_KEEP)
        except binding.FtError as e:
            assert e.code == fmt.FT_ECLOSED
            j1 = eng.submit(d1, [9], C, fmt.FT_OPEN | fmt.FT_KEEP)
        eng.wait(j1)
        eng.wait(j0)
        _images_equal(orc, eng)
        binding.job_release(eng.pool, j0)
        binding.job_release(eng.pool, j1)
        # a source outside every pageable window is refused
        bad = make_descs([dict(func=0, src_space=FT_PAGEABLE, dst_space=FT_POOL, src=48 * MiB - 8, dst=alloc(4096),
                               row_bytes=64)])
        with pytest.raises(binding.FtError) as ei:
            eng.submit(bad, [1], C, fmt.FT_OPEN)
        assert ei.value.code == fmt.FT_ERANGE
    finally:
        eng.close()


def test_merges_from_another_thread_while_the_open_job_is_waited_for(gpu):
    """ft_wait on an open job must not keep the pool's other calls out: one thread waits for the long
    job while this one merges small ones into it and waits for each."""
    import threading
    binding, _ = gpu
    orc, eng, rng = _engines(gpu, 160 * MiB, 256 * MiB, seed=41)
    try:
        C = 256 * KiB
        binding.set_batch(eng.pool, 4, 2)
        big = make_descs(_h2p_job(orc, eng, rng, [48 * MiB, 40 * MiB], 80 * MiB))
        smalls = [make_descs(_h2p_job(orc, eng, rng, [int(rng.integers(64 * KiB, 900 * KiB))], 80 * MiB)) for _ in range(12)]
        orc.wait(orc.submit(big, [1, 1], C))
        for d in smalls:
            orc.wait(orc.submit(d, [7], C))
        j0 = eng.submit(big, [1, 1], C, fmt.FT_OPEN | fmt.FT_TIMING)
        err = []

        def waiter():
            try:
                eng.wait(j0)
            except Exception as e:      # noqa: BLE001
                err.append(e)
        th = threading.Thread(target=waiter)
        th.start()
        merged = 0
        for d in smalls:
            try:
                j = eng.merge(j0, d, [7])
                merged += 1
            except binding.FtError as e:
                assert e.code == fmt.FT_ECLOSED
                j = eng.submit(d, [7], C, 0)
            eng.wait(j)
        th.join(timeout=60)
        assert not th.is_alive() and not err
        st = binding.job_stats(eng.pool, j0)
        assert st.cls[0].device_ms > 0 and st.cls[0].tickets > 0
        binding.job_release(eng.pool, j0)
        _images_equal(orc, eng)
        print(f"{merged} of {len(smalls)} merged while another thread waited", flush=True)
        assert merged >= 1
    finally:
        eng.close()


def test_closed_jobs_waited_for_from_several_threads(gpu):
    """ft_wait gives the pool's lock up while it blocks: four threads each wait for a job of their own
    while this thread keeps submitting; a kept job cannot be released under a waiter's feet."""
    import threading
    binding, _ = gpu
    orc, eng, rng = _engines(gpu, 200 * MiB, 320 * MiB, seed=43)
    try:
        C = 512 * KiB
        jobs = [make_descs(_h2p_job(orc, eng, rng, [int(rng.integers(6 * MiB, 20 * MiB)), 3 * MiB + 5], 100 * MiB))
                for _ in range(4)]
        late = [make_descs(_h2p_job(orc, eng, rng, [int(rng.integers(64 * KiB, 2 * MiB))], 100 * MiB)) for _ in range(6)]
        for d in jobs:
            orc.wait(orc.submit(d, [1, 3], C))
        for d in late:
            orc.wait(orc.submit(d, [2], C))
        handles = [eng.submit(d, [1, 3], C, fmt.FT_KEEP | fmt.FT_DETACHED) for d in jobs]
        err = []

        def waiter(j):
            try:
                eng.wait(j)
            except Exception as e:      # noqa: BLE001
                err.append(e)
        threads = [threading.Thread(target=waiter, args=(j,)) for j in handles]
        for th in threads:
            th.start()
        for d in late:
            eng.wait(eng.submit(d, [2], C, 0))
        for th in threads:
            th.join(timeout=60)
            assert not th.is_alive()
        assert not err, err
        for j in handles:
            with pytest.raises(binding.FtError) as ei:
                eng.wait(j)                      # a job is waited for once
            assert ei.value.code == fmt.FT_EINVAL
            binding.job_release(eng.pool, j)
        _images_equal(orc, eng)
    finally:
        eng.close()


def test_open_jobs_of_many_small_descriptors(gpu):
    """Functions made of hundreds of small transfers (several descriptors per tile, so the library
    keeps a descriptor entry per tile) in an open job, with a merge that rebuilds the order in the
    middle of the streams; pool->pool pieces at every alignment."""
    binding, _ = gpu
    orc, eng, rng = _engines(gpu, 96 * MiB, 160 * MiB, seed=47)
    try:
        C = 128 * KiB
        binding.set_batch(eng.pool, 3, 2)

        def many(nfunc, per_func, lo, hi, space):
            recs = []
            for f in range(nfunc):
                for _ in range(per_func):
                    n = int(rng.integers(lo, hi))
                    a = orc.slab_alloc(n + 32)
                    assert eng.slab_alloc(n + 32) == a
                    if space == FT_HOST:
                        src = int(rng.integers(0, 40 * MiB)) + int(rng.integers(0, 16))
                    else:
                        src = orc.slab_alloc(n + 32)
                        assert eng.slab_alloc(n + 32) == src
                        fill = rng.integers(0, 256, n + 32, dtype=np.uint8)
                        orc.write_pool(src, fill)
                        eng.write_pool(src, fill)
                        src += int(rng.integers(0, 16))
                    recs.append(dict(func=f, src_space=space, dst_space=FT_POOL, src=src,
                                     dst=a + int(rng.integers(0, 16)), row_bytes=n))
            return make_descs(recs)
        first = many(3, 260, 3000, 40000, FT_HOST)
        second = many(2, 150, 500, 9000, FT_HOST)
        third = many(2, 200, 2000, 30000, FT_POOL)
        orc.wait(orc.submit(first, [1, 2, 3], C))
        orc.wait(orc.submit(second, [5, 5], C))
        orc.wait(orc.submit(third, [1, 4], C))
        j0 = eng.submit(first, [1, 2, 3], C, fmt.FT_OPEN | fmt.FT_KEEP)
        try:
            j1 = eng.merge(j0, second, [5, 5], fmt.FT_KEEP)
            print("second job joined at batch", binding.job_arrival(eng.pool, j1, 0), flush=True)
        except binding.FtError as e:
            assert e.code == fmt.FT_ECLOSED
            j1 = eng.submit(second, [5, 5], C, fmt.FT_KEEP)
        j2 = eng.submit(third, [1, 4], C, fmt.FT_OPEN | fmt.FT_KEEP)   # an open pool->pool sequence of its own
        for j in (j2, j1, j0):
            eng.wait(j)
            binding.job_release(eng.pool, j)
        _images_equal(orc, eng)
    finally:
        eng.close()


@pytest.mark.parametrize("batch,depth,threads", [(5, 3, 4), (2, 1, 1), (4, 2, 3)])
def test_pageable_destinations_through_the_ring(gpu, batch, depth, threads):
    """Pool -> ordinary host memory: the device writes the pinned ring and the library's threads
    carry each finished batch on to its destination. Many more batches than slots, odd sizes and
    alignments, a pitched destination, pinned and pageable destinations in one function, a job in
    the other direction (pageable sources) in the same open sequence, a merge. Pageable memory,
    pinned memory and the pool must all be the oracle's afterwards."""
    from workloads import FT_PAGEABLE
    binding, _ = gpu
    orc, eng, rng = _engines(gpu, 64 * MiB, 192 * MiB, seed=29 + batch)
    try:
        C = 64 * KiB
        page = rng.integers(0, 256, 24 * MiB, dtype=np.uint8)
        for e in (orc, eng):
            e.pageable_arena(64 * MiB)
            e.write_pageable(0, page)          # lower part: sources; upper part keeps its fill: destinations
        binding.set_batch(eng.pool, batch, depth)
        binding.set_stage_threads(eng.pool, threads)

        def filled(n):
            a = orc.slab_alloc(n)
            assert eng.slab_alloc(n) == a
            data = rng.integers(0, 256, n, dtype=np.uint8)
            orc.write_pool(a, data)
            eng.write_pool(a, data)
            return a

        def alloc(n):
            a = orc.slab_alloc(n)
            assert eng.slab_alloc(n) == a
            return a
        out = 32 * MiB
        recs0 = [
            dict(func=0, src_space=FT_POOL, dst_space=FT_PAGEABLE, src=filled(8 * MiB) + 3, dst=out + 1, row_bytes=7 * MiB + 777),
            dict(func=1, src_space=FT_POOL, dst_space=FT_PAGEABLE, src=filled(3 * MiB), dst=out + 8 * MiB + 16, row_bytes=3 * MiB),
            # pinned and pageable destinations in one function's stream
            dict(func=1, src_space=FT_POOL, dst_space=FT_HOST, src=filled(1 * MiB) + 9, dst=40 * MiB + 5, row_bytes=600001),
            dict(func=1, src_space=FT_POOL, dst_space=FT_PAGEABLE, src=filled(4096), dst=out + 12 * MiB + 7, row_bytes=99),
            # packed rows of 200 bytes scattered at a pitch of 1000
            dict(func=2, src_space=FT_POOL, dst_space=FT_PAGEABLE, src=filled(2 * MiB) + 2, dst=out + 13 * MiB + 9,
                 row_bytes=200, rows=9000, src_pitch=200, dst_pitch=1000),
            # the other direction in the same job: a ring of its own
            dict(func=2, src_space=FT_PAGEABLE, dst_space=FT_POOL, src=5 * MiB + 1, dst=alloc(5 * MiB) + 4, row_bytes=4 * MiB + 5),
            dict(func=0, src_space=FT_POOL, dst_space=FT_POOL, src=filled(2 * MiB), dst=alloc(2 * MiB) + 1, row_bytes=2 * MiB - 9),
        ]
        recs1 = [dict(func=0, src_space=FT_POOL, dst_space=FT_PAGEABLE, src=filled(2 * MiB) + 1, dst=out + 24 * MiB + 3,
                      row_bytes=1 * MiB + 19)]
        d0, d1 = make_descs(recs0), make_descs(recs1)
        orc.wait(orc.submit(d0, [1, 2, 3], C))
        orc.wait(orc.submit(d1, [9], C))
        print(f"pageable destinations batch={batch} depth={depth} threads={threads}", flush=True)
        with pytest.raises(binding.FtError) as ei:
            eng.submit(d1, [9], C, fmt.FT_PATH_DMA)        # the comparison path has no way for pageable memory
        assert ei.value.code == fmt.FT_EINVAL
        j0 = eng.submit(d0, [1, 2, 3], C, fmt.FT_OPEN | fmt.FT_KEEP | fmt.FT_VALIDATE)
        try:
            j1 = eng.merge(j0, d1, [9], fmt.FT_KEEP)
        except binding.FtError as e:
            assert e.code == fmt.FT_ECLOSED
            j1 = eng.submit(d1, [9], C, fmt.FT_OPEN | fmt.FT_KEEP)
        eng.wait(j1)
        # the small job's bytes are at their destination when its own wait returns
        assert np.array_equal(eng.pageable_np[out + 24 * MiB + 3:out + 25 * MiB + 22],
                              orc.pageable_mem[out + 24 * MiB + 3:out + 25 * MiB + 22])
        eng.wait(j0)
        _images_equal(orc, eng)
        assert np.array_equal(eng.pageable_np, orc.pageable_mem), "pageable image differs"
        binding.job_release(eng.pool, j0)
        binding.job_release(eng.pool, j1)
        # refused: a destination outside every pageable window; host to host in any flavour
        for bad, code in ((dict(func=0, src_space=FT_POOL, dst_space=FT_PAGEABLE, src=filled(4096), dst=64 * MiB - 8,
                                row_bytes=64), fmt.FT_ERANGE),
                          (dict(func=0, src_space=FT_HOST, dst_space=FT_PAGEABLE, src=0, dst=out, row_bytes=64), fmt.FT_EINVAL),
                          (dict(func=0, src_space=FT_PAGEABLE, dst_space=FT_PAGEABLE, src=0, dst=out, row_bytes=64),
                           fmt.FT_EINVAL)):
            with pytest.raises(binding.FtError) as ei:
                eng.submit(make_descs([bad]), [1], C, fmt.FT_OPEN)
            assert ei.value.code == code
    finally:
        eng.close()


def test_pool_to_pool_open_job_triggers_larger_batches(gpu):
    """The on-device class puts 64 x batch_chunks chunks into a batch; the batches it triggers are the
    oracle's for that batch size, merged job included."""
    binding, _ = gpu
    orc, eng, rng = _engines(gpu, 4 * MiB, 256 * MiB, seed=53)
    try:
        C = 64 * KiB
        binding.set_batch(eng.pool, 2, 2)

        def job(sizes):
            recs = []
            for f, n in enumerate(sizes):
                a = orc.slab_alloc(n + 32)
                assert eng.slab_alloc(n + 32) == a
                b = orc.slab_alloc(n + 32)
                assert eng.slab_alloc(n + 32) == b
                data = rng.integers(0, 256, n + 32, dtype=np.uint8)
                orc.write_pool(a, data)
                eng.write_pool(a, data)
                recs.append(dict(func=f, src_space=FT_POOL, dst_space=FT_POOL, src=a + int(rng.integers(0, 16)),
                                 dst=b + int(rng.integers(0, 16)), row_bytes=n))
            return make_descs(recs)
        sizes0, w0 = [30 * MiB + 5, 22 * MiB, 9 * MiB + 4096], [1, 2, 1]
        sizes1, w1 = [3 * MiB + 7], [6]
        d0, d1 = job(sizes0), job(sizes1)
        orc.wait(orc.submit(d0, w0, C))
        orc.wait(orc.submit(d1, w1, C))
        j0 = eng.submit(d0, w0, C, fmt.FT_OPEN | fmt.FT_KEEP)
        spec = [{"n": [chunk_count(s, C) for s in sizes0], "w": w0}]
        index = {j0: 0}
        try:
            j1 = eng.merge(j0, d1, w1, fmt.FT_KEEP)
            spec.append({"n": [chunk_count(s, C) for s in sizes1], "w": w1, "arrive": binding.job_arrival(eng.pool, j1, 2)})
            index[j1] = 1
        except binding.FtError as e:
            assert e.code == fmt.FT_ECLOSED
            j1 = eng.submit(d1, w1, C, fmt.FT_KEEP)
        eng.wait(j1)
        eng.wait(j0)
        _images_equal(orc, eng)
        got = binding.job_batches(eng.pool, j0, 2)
        got = [[(index[j], f, k) for j, f, k in b] for b in got]
        assert got == batched_order(spec, 128)
        assert max(len(b) for b in got) == 128
        print("pool->pool batches", len(got), "arrivals", [s.get("arrive", 0) for s in spec], flush=True)
        binding.job_release(eng.pool, j0)
        binding.job_release(eng.pool, j1)
    finally:
        eng.close()


def test_two_pools_driven_from_two_threads(gpu):
    """Two pools on one device share its streams, table buffers, events and counter pairs. Two threads
    run twenty jobs each (small ones that travel with the launch, larger ones with uploaded tables, an
    open job with a merge) at the same time; each pool's memory must be its own oracle's."""
    import threading
    binding, harness = gpu
    pairs = []
    for t in range(2):
        orc, eng, rng = _engines(gpu, 48 * MiB, 128 * MiB, seed=61 + t)
        pairs.append((orc, eng, rng))
    err = []

    def work(t):
        orc, eng, rng = pairs[t]
        try:
            for i in range(20):
                kind = i % 4
                sizes = [[int(rng.integers(1, 200000))], [int(rng.integers(1 * MiB, 3 * MiB)), 70001],
                         [5 * MiB + 3, 2 * MiB], [int(rng.integers(64 * KiB, 900 * KiB))]][kind]
                d = make_descs(_h2p_job(orc, eng, rng, sizes, 24 * MiB))
                w = [1 + (i + f) % 3 for f in range(len(sizes))]
                orc.wait(orc.submit(d, w, 256 * KiB))
                if kind == 2:
                    extra = make_descs(_h2p_job(orc, eng, rng, [300001], 24 * MiB))
                    orc.wait(orc.submit(extra, [4], 256 * KiB))
                    j0 = eng.submit(d, w, 256 * KiB, fmt.FT_OPEN)
                    try:
                        j1 = eng.merge(j0, extra, [4])
                    except binding.FtError as e:
                        assert e.code == fmt.FT_ECLOSED
                        j1 = eng.submit(extra, [4], 256 * KiB, 0)
                    eng.wait(j1)
                    eng.wait(j0)
                else:
                    eng.wait(eng.submit(d, w, 256 * KiB, fmt.FT_DETACHED if kind == 1 else 0))
        except Exception as e:      # noqa: BLE001
            err.append((t, repr(e)))
    try:
        threads = [threading.Thread(target=work, args=(t,)) for t in range(2)]
        for th in threads:
            th.start()
        for th in threads:
            th.join(timeout=120)
            assert not th.is_alive()
        assert not err, err
        for orc, eng, _ in pairs:
            _images_equal(orc, eng)
    finally:
        for _, eng, _ in pairs:
            eng.close()


def _random_open_sequences(gpu, seeds):
    from workloads import FT_PAGEABLE
    binding, _ = gpu
    for seed in seeds:
        orc, eng, rng = _engines(gpu, 64 * MiB, 256 * MiB, seed=seed)
        pyr = __import__("random").Random(seed)
        try:
            page = rng.integers(0, 256, 24 * MiB, dtype=np.uint8)
            for e in (orc, eng):
                e.pageable_arena(48 * MiB)
                e.write_pageable(0, page)
            hdst = [40 * MiB]          # pinned destinations
            pdst = [24 * MiB]          # pageable destinations

            def job(nfunc):
                recs = []
                for _ in range(pyr.choice([1, 2, 3, 5])):
                    kind = pyr.choice(["h2p", "h2p", "pg2p", "p2h", "p2pg", "p2p"])
                    rows = pyr.choice([1, 1, 1, 7, 300])
                    rb = pyr.choice([33, 4096, 250001, 1 * MiB + 3, 3 * MiB]) if rows == 1 else pyr.choice([48, 200, 1000])
                    sp, dp = rb + pyr.choice([0, 8, 100]), rb + pyr.choice([0, 0, 24])
                    es, ed = (rows - 1) * sp + rb, (rows - 1) * dp + rb
                    if kind in ("h2p", "pg2p"):
                        src = pyr.randrange(0, 20 * MiB - es)
                        sspace = FT_HOST if kind == "h2p" else FT_PAGEABLE
                    else:
                        a = orc.slab_alloc(es + 32)
                        assert eng.slab_alloc(es + 32) == a
                        fill = rng.integers(0, 256, es + 32, dtype=np.uint8)
                        orc.write_pool(a, fill)
                        eng.write_pool(a, fill)
                        src, sspace = a + pyr.randrange(16), FT_POOL
                    if kind == "p2h":
                        dst, dspace = hdst[0] + pyr.randrange(16), FT_HOST
                        hdst[0] += (ed + 47) // 16 * 16
                    elif kind == "p2pg":
                        dst, dspace = pdst[0] + pyr.randrange(16), FT_PAGEABLE
                        pdst[0] += (ed + 47) // 16 * 16
                    else:
                        b = orc.slab_alloc(ed + 32)
                        assert eng.slab_alloc(ed + 32) == b
                        dst, dspace = b + pyr.randrange(16), FT_POOL
                    assert hdst[0] < 62 * MiB and pdst[0] < 46 * MiB
                    recs.append(dict(func=pyr.randrange(nfunc), src_space=sspace, dst_space=dspace, src=src, dst=dst,
                                     row_bytes=rb, rows=rows, src_pitch=sp, dst_pitch=dp))
                return make_descs(recs)
            for rnd in range(4):
                C = pyr.choice([64 * KiB, 256 * KiB])
                binding.set_batch(eng.pool, pyr.choice([1, 2, 5]), pyr.choice([1, 2, 3]))
                binding.set_stage_threads(eng.pool, pyr.choice([1, 2, 4]))
                nf0 = pyr.choice([1, 2, 4])
                w0 = [pyr.choice([1, 2, 5]) for _ in range(nf0)]
                d0 = job(nf0)
                later = []
                for _ in range(pyr.choice([0, 1, 3])):
                    nf = pyr.choice([1, 2])
                    later.append((job(nf), [pyr.choice([1, 3, 9]) for _ in range(nf)]))
                orc.wait(orc.submit(d0, w0, C))
                for d, w in later:
                    orc.wait(orc.submit(d, w, C))
                handles = [eng.submit(d0, w0, C, fmt.FT_OPEN | (fmt.FT_VALIDATE if rnd % 2 else 0))]
                for d, w in later:
                    try:
                        handles.append(eng.merge(handles[0], d, w))
                    except binding.FtError as e:
                        assert e.code == fmt.FT_ECLOSED, e.code
                        handles.append(eng.submit(d, w, C, fmt.FT_OPEN))
                # weights changed at random moments: whatever order results, the bytes are the plain copy
                nfuncs = [nf0] + [len(w) for _, w in later]
                for _ in range(pyr.choice([0, 1, 3])):
                    i = pyr.randrange(len(handles))
                    try:
                        binding.job_reweight(eng.pool, handles[i], [pyr.choice([1, 2, 11]) for _ in range(nfuncs[i])])
                    except binding.FtError as e:      # a later job that ran on its own as a closed job
                        assert e.code == fmt.FT_EINVAL, e.code
                pyr.shuffle(handles)
                for h in handles:
                    eng.wait(h)
                _images_equal(orc, eng)
                assert np.array_equal(eng.pageable_np, orc.pageable_mem), (seed, rnd)
            print(f"random open sequences seed={seed} done", flush=True)
        finally:
            eng.close()


def test_random_open_jobs_with_merges_and_both_rings(gpu):
    """Random open jobs (pinned and pageable host sides in both directions, pool->pool, pitched pieces, any
    alignment), random batch size, depth and staging threads, up to three later jobs merged while each runs
    (or started on their own when the open one has already closed), waited for in random order."""
    _random_open_sequences(gpu, (301, 302, 303))


@pytest.mark.parametrize("batch,depth", [(5, 2), (2, 1)])
def test_weights_changed_while_the_sequence_runs(gpu, batch, depth):
    """Sec. 6.1's rate control on a running sequence: a long host->pool job, a second one merged, then the
    weights of both changed (the first one twice). The library says from which batch each change holds;
    with those counts the batches must be the oracle's, and the bytes the plain copy whatever the order."""
    binding, _ = gpu
    orc, eng, rng = _engines(gpu, 192 * MiB, 256 * MiB, seed=40 + batch)
    try:
        C = 256 * KiB
        binding.set_batch(eng.pool, batch, depth)
        jobs_sizes = [[48 * MiB, 30 * MiB + 48, 11 * MiB + 5], [6 * MiB + 7, 5 * MiB]]
        jobs_w = [[1, 1, 1], [2, 2]]
        descs = [make_descs(_h2p_job(orc, eng, rng, s, 96 * MiB)) for s in jobs_sizes]
        for d, w in zip(descs, jobs_w):
            orc.wait(orc.submit(d, w, C))
        print(f"reweight batch={batch} depth={depth}", flush=True)
        handles = [eng.submit(descs[0], jobs_w[0], C, fmt.FT_OPEN | fmt.FT_KEEP)]
        changes = {0: [], 1: []}
        at = binding.job_reweight(eng.pool, handles[0], [1, 6, 1])
        assert at[1] is None and at[2] is None
        if at[0] is not None:
            changes[0].append((at[0], [1, 6, 1]))
        merged = True
        try:
            handles.append(eng.merge(handles[0], descs[1], jobs_w[1], fmt.FT_KEEP))
        except binding.FtError as e:
            assert e.code == fmt.FT_ECLOSED
            merged = False
            handles.append(eng.submit(descs[1], jobs_w[1], C, fmt.FT_KEEP))
        time.sleep(0.0003)
        for j, w in ((1, [9, 1]), (0, [3, 1, 7])):
            if j == 1 and not merged:
                continue
            at = binding.job_reweight(eng.pool, handles[j], w)
            if at[0] is not None:
                changes[j].append((at[0], w))
        # bad arguments change nothing
        for bad in ([1, 2], [1, 0, 1]):
            with pytest.raises(binding.FtError) as err:
                binding.job_reweight(eng.pool, handles[0], bad)
            assert err.value.code == fmt.FT_EINVAL
        for h in handles:
            eng.wait(h)
        _images_equal(orc, eng)
        spec = [{"n": [chunk_count(s, C) for s in jobs_sizes[0]], "w": jobs_w[0], "reweight": changes[0]}]
        index = {handles[0]: 0}
        if merged:
            index[handles[1]] = 1
            spec.append({"n": [chunk_count(s, C) for s in jobs_sizes[1]], "w": jobs_w[1],
                         "arrive": binding.job_arrival(eng.pool, handles[1], 0), "reweight": changes[1]})
        got = binding.job_batches(eng.pool, handles[0], 0)
        got = [[(index[j], f, k) for j, f, k in b] for b in got]
        assert got == batched_order(spec, batch)
        print("changes", changes, "merged", merged, "batches", len(got), flush=True)
        # once everything is triggered a change is accepted and reports that nothing is left
        assert binding.job_reweight(eng.pool, handles[0], [1, 1, 1]) == [None, None, None]
        for h in handles:
            binding.job_release(eng.pool, h)
        # a closed job is not part of a sequence
        d = make_descs(_h2p_job(orc, eng, rng, [300 * KiB], 96 * MiB))
        orc.wait(orc.submit(d, [1], C))
        plain = eng.submit(d, [1], C)
        with pytest.raises(binding.FtError) as err:
            binding.job_reweight(eng.pool, plain, [2])
        assert err.value.code == fmt.FT_EINVAL
        eng.wait(plain)
    finally:
        eng.close()


def test_weights_changed_on_every_class_at_once(gpu):
    """One open job with host->pool, pool->host and pool->pool functions, reweighted while it runs: each
    class reports its own batch, each class's batches are the oracle's for that count."""
    binding, _ = gpu
    orc, eng, rng = _engines(gpu, 160 * MiB, 512 * MiB, seed=77)
    try:
        C = 256 * KiB
        binding.set_batch(eng.pool, 4, 2)
        sizes = [20 * MiB, 12 * MiB + 40, 18 * MiB, 9 * MiB + 8, 96 * MiB, 64 * MiB + 16]
        recs, hdst = [], 80 * MiB
        for f, n in enumerate(sizes):
            a = orc.slab_alloc(n + 32)
            assert eng.slab_alloc(n + 32) == a
            if f < 2:
                recs.append(dict(func=f, src_space=FT_HOST, dst_space=FT_POOL, src=f * 24 * MiB + 3 * f, dst=a + 5,
                                 row_bytes=n))
                continue
            fill = rng.integers(0, 256, n + 32, dtype=np.uint8)
            orc.write_pool(a, fill)
            eng.write_pool(a, fill)
            if f < 4:
                recs.append(dict(func=f, src_space=FT_POOL, dst_space=FT_HOST, src=a + 1, dst=hdst + 7, row_bytes=n))
                hdst += 24 * MiB
            else:
                b = orc.slab_alloc(n + 32)
                assert eng.slab_alloc(n + 32) == b
                recs.append(dict(func=f, src_space=FT_POOL, dst_space=FT_POOL, src=a + 2, dst=b + 9, row_bytes=n))
        d = make_descs(recs)
        w0, w1 = [1, 1, 1, 1, 1, 1], [1, 5, 4, 1, 2, 7]
        orc.wait(orc.submit(d, w0, C))
        job = eng.submit(d, w0, C, fmt.FT_OPEN | fmt.FT_KEEP)
        w2 = [3, 1, 1, 6, 5, 1]
        at = binding.job_reweight(eng.pool, job, w1)
        time.sleep(0.0003)
        at2 = binding.job_reweight(eng.pool, job, w2)
        eng.wait(job)
        _images_equal(orc, eng)
        print("reweighted at", at, "and", at2, flush=True)
        for c, fs, B in ((0, (0, 1), 4), (1, (2, 3), 4), (2, (4, 5), 256)):
            spec = {"n": [chunk_count(sizes[f], C) for f in fs], "w": [w0[f] for f in fs], "reweight": []}
            for when, w in ((at[c], w1), (at2[c], w2)):
                if when is not None:
                    spec["reweight"].append((when, [w[f] for f in fs]))
            got = binding.job_batches(eng.pool, job, c)
            got = [[(fs.index(f), k) for _, f, k in b] for b in got]
            assert got == [[(f, k) for _, f, k in b] for b in batched_order([spec], B)], c
        binding.job_release(eng.pool, job)
    finally:
        eng.close()


def test_pool_destroyed_with_open_jobs_in_flight(gpu):
    """ft_pool_destroy waits for everything: an open job with all three classes and a pageable destination,
    a job merged into it, a closed job - none of them waited for - and every byte is where it belongs
    when the call returns."""
    from workloads import FT_PAGEABLE
    binding, _ = gpu
    orc, eng, rng = _engines(gpu, 128 * MiB, 256 * MiB, seed=91)
    try:
        C = 256 * KiB
        for e in (orc, eng):
            e.pageable_arena(16 * MiB)
        binding.set_batch(eng.pool, 3, 2)

        def alloc(n):
            a = orc.slab_alloc(n)
            assert eng.slab_alloc(n) == a
            return a

        def filled(n):
            a = alloc(n)
            data = rng.integers(0, 256, n, dtype=np.uint8)
            orc.write_pool(a, data)
            eng.write_pool(a, data)
            return a

        big = 20 * MiB
        recs0 = [dict(func=0, src_space=FT_HOST, dst_space=FT_POOL, src=8192 + 1, dst=alloc(big) + 2, row_bytes=big - 16),
                 dict(func=1, src_space=FT_POOL, dst_space=FT_HOST, src=filled(big), dst=64 * MiB + 3, row_bytes=big),
                 dict(func=2, src_space=FT_POOL, dst_space=FT_POOL, src=filled(big) + 5, dst=alloc(big), row_bytes=big - 16),
                 dict(func=1, src_space=FT_POOL, dst_space=FT_PAGEABLE, src=filled(6 * MiB), dst=4096 + 7, row_bytes=6 * MiB)]
        recs1 = [dict(func=0, src_space=FT_HOST, dst_space=FT_POOL, src=30 * MiB, dst=alloc(3 * MiB), row_bytes=3 * MiB)]
        recs2 = [dict(func=0, src_space=FT_POOL, dst_space=FT_POOL, src=filled(5 * MiB), dst=alloc(5 * MiB) + 1,
                      row_bytes=5 * MiB - 1)]
        d0, d1, d2 = make_descs(recs0), make_descs(recs1), make_descs(recs2)
        for d, w in ((d0, [1, 2, 1]), (d1, [4]), (d2, [1])):
            orc.wait(orc.submit(d, w, C))
        j0 = eng.submit(d0, [1, 2, 1], C, fmt.FT_OPEN)
        try:
            eng.merge(j0, d1, [4])
        except binding.FtError as e:
            assert e.code == fmt.FT_ECLOSED
            eng.submit(d1, [4], C, fmt.FT_DETACHED)
        eng.submit(d2, [1], C, fmt.FT_DETACHED)
        segments = list(eng.segments)
        print("destroying the pool with three jobs in flight", flush=True)
        binding.pool_destroy(eng.pool)          # no ft_wait before it
        eng.pool = None
        import torch
        assert np.array_equal(eng.host_np[:len(orc.host_mem)], orc.host_mem), "host image differs"
        assert np.array_equal(eng.pageable_np, orc.pageable_mem), "pageable image differs"
        got = torch.cat([t for t, _ in segments]).cpu().numpy()
        assert np.array_equal(got, orc.pool_mem), "pool image differs"
    finally:
        eng.close()


def test_closed_jobs_with_little_pageable_memory(gpu):
    """Without FT_OPEN up to 8 MiB of pageable memory go through a pinned buffer of the job's own: sources are
    taken when the job is submitted, destinations are complete when ft_wait returns. Small and larger jobs (both
    launch routes), pitched and plain, both directions mixed with pinned and pool->pool pieces, several jobs in
    flight at once; more than 8 MiB is refused."""
    from workloads import FT_PAGEABLE
    binding, _ = gpu
    orc, eng, rng = _engines(gpu, 32 * MiB, 128 * MiB, seed=61)
    pyr = __import__("random").Random(61)
    try:
        page = rng.integers(0, 256, 12 * MiB, dtype=np.uint8)
        for e in (orc, eng):
            e.pageable_arena(32 * MiB)
            e.write_pageable(0, page)
        pdst = [16 * MiB]
        pending = []
        for case in range(40):
            recs = []
            for _ in range(pyr.choice([1, 1, 2, 4])):
                kind = pyr.choice(["pg2p", "pg2p", "p2pg", "p2pg", "h2p", "p2p"])
                rows = pyr.choice([1, 1, 3, 60])
                rb = pyr.choice([1, 100, 4096, 70001, 900 * KiB]) if rows == 1 else pyr.choice([5, 64, 300, 2000])
                sp, dp = rb + pyr.choice([0, 0, 8, 100]), rb + pyr.choice([0, 0, 24])
                es, ed = (rows - 1) * sp + rb, (rows - 1) * dp + rb
                if kind in ("pg2p", "h2p"):
                    src, sspace = pyr.randrange(0, 10 * MiB - es), FT_PAGEABLE if kind == "pg2p" else FT_HOST
                else:
                    a = orc.slab_alloc(es + 32)
                    assert eng.slab_alloc(es + 32) == a
                    fill = rng.integers(0, 256, es + 32, dtype=np.uint8)
                    orc.write_pool(a, fill)
                    eng.write_pool(a, fill)
                    src, sspace = a + pyr.randrange(16), FT_POOL
                if kind == "p2pg":
                    dst, dspace = pdst[0] + pyr.randrange(16), FT_PAGEABLE
                    pdst[0] += (ed + 47) // 16 * 16
                    assert pdst[0] < 31 * MiB
                else:
                    b = orc.slab_alloc(ed + 32)
                    assert eng.slab_alloc(ed + 32) == b
                    dst, dspace = b + pyr.randrange(16), FT_POOL
                recs.append(dict(func=pyr.randrange(2), src_space=sspace, dst_space=dspace, src=src, dst=dst,
                                 row_bytes=rb, rows=rows, src_pitch=sp, dst_pitch=dp))
            d = make_descs(recs)
            w = [pyr.choice([1, 3]), pyr.choice([1, 2])]
            C = pyr.choice([64 * KiB, 2 * MiB])
            orc.wait(orc.submit(d, w, C))
            pending.append(eng.submit(d, w, C, pyr.choice([0, fmt.FT_DETACHED, fmt.FT_VALIDATE])))
            if len(pending) == 3 or case == 39:
                # pageable sources were taken at submit: overwriting them now changes nothing
                for h in pending:
                    eng.wait(h)
                pending = []
                _images_equal(orc, eng)
                assert np.array_equal(eng.pageable_np, orc.pageable_mem), case
        print("closed pageable jobs done", flush=True)
        # rings taken ahead of time serve the open jobs that follow (and the call can be repeated)
        binding.set_batch(eng.pool, 3, 2)
        binding.reserve_rings(eng.pool, 256 * KiB)
        binding.reserve_rings(eng.pool, 256 * KiB)
        with pytest.raises(binding.FtError) as ei:
            binding.reserve_rings(eng.pool, 100)
        assert ei.value.code == fmt.FT_EINVAL
        # sources are free again as soon as the submit has returned
        n = 300 * KiB
        a = orc.slab_alloc(n)
        assert eng.slab_alloc(n) == a
        d = make_descs([dict(func=0, src_space=FT_PAGEABLE, dst_space=FT_POOL, src=0, dst=a, row_bytes=n)])
        orc.wait(orc.submit(d, [1], 2 * MiB))
        h = eng.submit(d, [1], 2 * MiB)
        eng.pageable_np[:n] ^= 0xFF                        # only on the engine's side
        eng.wait(h)
        eng.pageable_np[:n] ^= 0xFF
        _images_equal(orc, eng)
        # too much for the buffer: an open job is the way
        big = 9 * MiB
        b = orc.slab_alloc(big)
        assert eng.slab_alloc(big) == b
        d = make_descs([dict(func=0, src_space=FT_PAGEABLE, dst_space=FT_POOL, src=0, dst=b, row_bytes=big)])
        with pytest.raises(binding.FtError) as ei:
            eng.submit(d, [1], 2 * MiB)
        assert ei.value.code == fmt.FT_EINVAL
        orc.wait(orc.submit(d, [1], 2 * MiB))
        eng.wait(eng.submit(d, [1], 2 * MiB, fmt.FT_OPEN))
        _images_equal(orc, eng)
    finally:
        eng.close()
