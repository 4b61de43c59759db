"""Full-size workloads in the launch configuration bench.py times (default launch
shapes, large_mixed submitted detached), checked by what holds at any size:

  * every destination range equals its source range (compared on the device or, for
    host memory, after one copy back) - the plain definition of the result;
  * sampled descriptors one by one against the CPU oracle on a re-based copy of just
    their source and destination windows (canary padding included);
  * the device's ticket order of every job and class equals the oracle's order;
  * allocation offsets and pool growth equal the oracle pool's.
"""
import numpy as np
import pytest

import oracle
from oracle import OracleEngine, stride_order, chunk_count
from workloads import configs, runner, make_descs, FT_HOST, FT_POOL
from workloads import format as fmt

pytestmark = pytest.mark.gpu

PAD = 64


def _class_of(d):
    return 0 if d["src_space"] == FT_HOST else (1 if d["dst_space"] == FT_HOST else 2)


def _view(eng, space, off, n):
    """uint8 tensor view of n bytes at `off` of the host arena or the pool."""
    if space == FT_HOST:
        return eng.host[off:off + n]
    t, o = eng._locate(off)
    return t[o:o + n]


def _rows(eng, d, side):
    space = int(d[side + "_space"])
    rows, rb = int(d["rows"]), int(d["row_bytes"])
    pitch = int(d[side + "_pitch"]) if rows > 1 else rb
    ext = (rows - 1) * pitch + rb
    v = _view(eng, space, int(d[side]), ext)
    if rows == 1:
        return v
    return v.as_strided((rows, rb), (pitch, 1))


def _oracle_one(eng, d):
    """Run one descriptor through the oracle on re-based windows and compare the
    destination window (with PAD bytes either side) with what the device holds."""
    rows, rb = int(d["rows"]), int(d["row_bytes"])
    sp = int(d["src_pitch"]) if rows > 1 else rb
    dp = int(d["dst_pitch"]) if rows > 1 else rb
    es, ed = (rows - 1) * sp + rb, (rows - 1) * dp + rb
    src_bytes = _view(eng, int(d["src_space"]), int(d["src"]), es).cpu().numpy()
    dst_lo = max(0, int(d["dst"]) - PAD)
    lead = int(d["dst"]) - dst_lo
    got = _view(eng, int(d["dst_space"]), dst_lo, lead + ed + PAD).cpu().numpy()
    orc = OracleEngine()
    slab = 4096
    orc.host_arena(((es + ed + 4 * PAD) // slab + 2) * slab)
    orc.pool_create(((es + ed + 4 * PAD) // slab + 2) * slab * 2, slab)
    a = orc.slab_alloc(es)
    b = orc.slab_alloc(lead + ed + PAD)
    # the destination window starts as the device's window looked before the job,
    # except inside the rows, which the job overwrites anyway
    orc.write_pool(b, got)
    orc.write_pool(a, src_bytes)
    one = make_descs([dict(func=0, src_space=FT_POOL, dst_space=FT_POOL, src=a, dst=b + lead,
                           row_bytes=rb, rows=rows, src_pitch=sp, dst_pitch=dp)])
    orc.wait(orc.submit(one, [1], 4096))
    want = orc.read_pool(b, lead + ed + PAD)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("name", ["tiny", "traffic", "feature", "contended", "large_mixed"])
def test_full_size_workload(name):
    import torch
    from paper_2411_01830_amd import binding as ft, harness
    print(f"full-size case {name}", flush=True)
    plan = configs.CONFIGS[name](1.0)
    # the oracle's pool bookkeeping alone (no memory image at this size)
    pool = oracle.Pool(plan.pool_bytes, plan.slab_bytes)
    want_off, total, targets, grows = {}, plan.pool_bytes, list(plan.grow_to), []
    for st in plan.steps:
        if st[0] != "alloc":
            continue
        while True:
            try:
                want_off[st[1]] = pool.alloc(st[2])
                break
            except oracle.OracleError as e:
                assert e.code == oracle.ENOMEM
                t = targets.pop(0)
                pool.grow(t - total)
                grows.append(t - total)
                total = t
    eng = harness.GpuEngine()
    flags = ft.FT_KEEP | (ft.FT_DETACHED if name == "large_mixed" else 0)
    try:
        rec = runner.run_plan(plan, eng, flags=flags)
        torch.cuda.synchronize()
        assert rec.alloc_off == want_off
        assert rec.grows == grows
        rng = np.random.default_rng(5)
        for jname, arr in rec.descs.items():
            # (1) every destination equals its source
            for d in arr:
                s, t = _rows(eng, d, "src"), _rows(eng, d, "dst")
                if s.device != t.device:
                    s, t = s.cpu(), t.cpu()
                assert torch.equal(s, t), (jname, int(d["src"]), int(d["dst"]))
            # (2) sampled descriptors through the oracle: odd alignments, extremes, random
            sizes = arr["row_bytes"].astype(np.int64) * arr["rows"].astype(np.int64)
            odd = np.flatnonzero(((arr["src"] - arr["dst"]) % 16 != 0) & (sizes < (8 << 20)))
            pick = set(odd[:6].tolist()) | {int(np.argmin(sizes))}
            small = np.flatnonzero(sizes < (8 << 20))
            pick |= set(rng.choice(small, size=min(6, len(small)), replace=False).tolist())
            for i in sorted(pick):
                _oracle_one(eng, arr[i])
            # (3) the device's ticket order
            w = rec.weights[jname]
            C = rec.chunk_bytes[jname]
            for cls in (0, 1, 2):
                S = [0] * len(w)
                for d in arr:
                    if _class_of(d) == cls:
                        S[int(d["func"])] += int(d["row_bytes"]) * int(d["rows"])
                want = stride_order([chunk_count(x, C) for x in S], w)
                assert eng.job_schedule(rec.jobs[jname], cls) == want, (jname, cls)
            ft.job_release(eng.pool, rec.jobs[jname])
    finally:
        eng.close()


@pytest.mark.parametrize("route", ["launch_argument", "uploaded_tables"])
def test_transfers_larger_than_four_gib(route):
    """Maximum sizes: one contiguous transfer of more than 4 GiB at unlike alignments and a pitched one
    whose extent passes 4 GiB, so every offset, stream position and pitch product needs its upper 32
    bits. Checked on the device by the definition of the result (destination rows equal source rows,
    canaries either side untouched), and the ticket order against the oracle's order."""
    import torch
    from paper_2411_01830_amd import binding as ft
    GiB = 1 << 30
    n1 = 4 * GiB + 123457
    rows, rb, sp, dp = 5, GiB + 48, GiB + 4096, GiB + 1000
    slab = 1 << 20
    need = lambda n: (n + slab - 1) // slab * slab
    sizes = [need(n1 + 64), need(n1 + 64), need((rows - 1) * sp + rb + 64), need((rows - 1) * dp + rb + 64)]
    total = sum(sizes)
    buf = torch.empty(total, dtype=torch.uint8, device="cuda:0")
    g = torch.Generator(device="cuda:0")
    g.manual_seed(4242)
    step = 1 << 28
    for o in range(0, total, step):
        m = min(step, total - o)
        buf[o:o + m] = torch.randint(0, 256, (m,), dtype=torch.uint8, device="cuda:0", generator=g)
    pool = ft.pool_create(buf.data_ptr(), total, slab, 0)
    try:
        a, b, c, d = (ft.slab_alloc(pool, s) for s in sizes)
        buf[b:b + sizes[1]] = 0xA5
        buf[d:d + sizes[3]] = 0xA5
        descs = make_descs([
            dict(func=0, src_space=FT_POOL, dst_space=FT_POOL, src=a + 3, dst=b + 9, row_bytes=n1),
            dict(func=1, src_space=FT_POOL, dst_space=FT_POOL, src=c + 5, dst=d + 16, row_bytes=rb, rows=rows,
                 src_pitch=sp, dst_pitch=dp)])
        flags = ft.FT_KEEP | (ft.FT_DETACHED if route == "uploaded_tables" else 0)
        chunk = 2 << 20
        w = [1, 3]
        print(f"huge transfers, route {route}", flush=True)
        job = ft.submit_transfers(pool, descs, w, chunk, flags, torch.cuda.current_stream().cuda_stream)
        ft.wait(pool, job)
        st = ft.job_stats(pool, job)
        assert st.cls[2].payload_bytes == n1 + rows * rb
        assert st.cls[2].in_launch == (1 if route == "launch_argument" else 0)
        assert torch.equal(buf[b + 9:b + 9 + n1], buf[a + 3:a + 3 + n1])
        assert bool((buf[b:b + 9] == 0xA5).all()) and bool((buf[b + 9 + n1:b + 9 + n1 + 55] == 0xA5).all())
        for r in range(rows):
            assert torch.equal(buf[d + 16 + r * dp:d + 16 + r * dp + rb], buf[c + 5 + r * sp:c + 5 + r * sp + rb]), r
            gap_end = d + 16 + (r + 1) * dp if r + 1 < rows else d + 16 + r * dp + rb + 48
            assert bool((buf[d + 16 + r * dp + rb:gap_end] == 0xA5).all()), r
        assert bool((buf[d:d + 16] == 0xA5).all())
        n = [chunk_count(n1, chunk), chunk_count(rows * rb, chunk)]
        assert ft.job_schedule(pool, job, 2) == stride_order(n, w)
        ft.job_release(pool, job)
    finally:
        ft.pool_destroy(pool)
        del buf
        torch.cuda.empty_cache()


def test_one_aligned_tensor_larger_than_four_gib():
    """The route on which the workgroups deal the tiles of one aligned tensor out among themselves, beyond 4 GiB:
    tile numbers times tile bytes need their upper 32 bits. Destination against source on the device, canaries either
    side; a length that leaves a ragged last tile."""
    import torch
    from paper_2411_01830_amd import binding as ft
    GiB = 1 << 30
    n = 4 * GiB + 5 * (1 << 20) + 4096 + 48
    slab = 1 << 20
    size = (n + 64 + slab - 1) // slab * slab
    buf = torch.empty(2 * size, dtype=torch.uint8, device="cuda:0")
    g = torch.Generator(device="cuda:0")
    g.manual_seed(4343)
    step = 1 << 28
    for o in range(0, size, step):
        m = min(step, size - o)
        buf[o:o + m] = torch.randint(0, 256, (m,), dtype=torch.uint8, device="cuda:0", generator=g)
    buf[size:] = 0xA5
    pool = ft.pool_create(buf.data_ptr(), 2 * size, slab, 0)
    try:
        a, b = ft.slab_alloc(pool, size), ft.slab_alloc(pool, size)
        d = make_descs([dict(func=0, src_space=FT_POOL, dst_space=FT_POOL, src=a + 16, dst=b + 32, row_bytes=n)])
        print("one aligned tensor beyond 4 GiB", flush=True)
        job = ft.submit_transfers(pool, d, [1], 2 << 20, ft.FT_KEEP, torch.cuda.current_stream().cuda_stream)
        ft.wait(pool, job)
        st = ft.job_stats(pool, job)
        assert st.cls[2].in_launch == 1 and st.cls[2].workgroups < st.cls[2].tickets
        assert torch.equal(buf[b + 32:b + 32 + n], buf[a + 16:a + 16 + n])
        assert bool((buf[b:b + 32] == 0xA5).all()) and bool((buf[b + 32 + n:b + size] == 0xA5).all())
        ft.job_release(pool, job)
    finally:
        ft.pool_destroy(pool)
        del buf
        torch.cuda.empty_cache()
