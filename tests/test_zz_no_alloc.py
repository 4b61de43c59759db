"""ft_submit_static, the submit that allocates nothing, against ft_submit_transfers and the oracle.

Two calls in a row on one stream with no synchronisation between them, the second with a smaller
input: the library's fixed device array keeps what the first call left in it, so the second call
must clear and overwrite what it uses. Bit-exact, as for every other path.
"""
import numpy as np
import pytest

from oracle import OracleEngine
from workloads import make_descs, FT_HOST, FT_POOL
from workloads import format as fmt

pytestmark = pytest.mark.gpu


def _engines(host, pool, slab, seed):
    from paper_2411_01830_amd import harness
    orc, a, b = OracleEngine(), harness.GpuEngine(), harness.GpuEngine()
    rng = np.random.default_rng(seed)
    data = rng.integers(0, 256, host // 2, dtype=np.uint8)
    for e in (orc, a, b):
        e.host_arena(host)
        e.pool_create(pool, slab)
        e.write_host(0, data)
    return orc, a, b, rng


def _alloc(engs, n, rng=None):
    off = engs[0].slab_alloc(n)
    for e in engs[1:]:
        assert e.slab_alloc(n) == off
    if rng is not None:
        fill = rng.integers(0, 256, n, dtype=np.uint8)
        for e in engs:
            e.write_pool(off, fill)
    return off


def _job(engs, rng, nfunc, per_func, sizes, host_dst_at):
    """A job with all three link classes: contiguous pieces at any alignment and pitched pieces."""
    recs = []
    for f in range(nfunc):
        for k in range(per_func):
            n = int(rng.integers(sizes[0], sizes[1]))
            kind = (f + k) % 4
            sa, da = int(rng.integers(0, 16)), int(rng.integers(0, 16))
            if kind == 0:      # host -> pool
                dst = _alloc(engs, n + 32)
                recs.append(dict(func=f, src_space=FT_HOST, dst_space=FT_POOL, src=4096 * int(rng.integers(0, 200)) + sa,
                                 dst=dst + da, row_bytes=n))
            elif kind == 1:    # pool -> host
                src = _alloc(engs, n + 32, rng)
                recs.append(dict(func=f, src_space=FT_POOL, dst_space=FT_HOST, src=src + sa, dst=host_dst_at[0] + da,
                                 row_bytes=n))
                host_dst_at[0] += (n + 64 + 15) // 16 * 16
            elif kind == 2:    # pool -> pool, contiguous
                src, dst = _alloc(engs, n + 32, rng), _alloc(engs, n + 32)
                recs.append(dict(func=f, src_space=FT_POOL, dst_space=FT_POOL, src=src + sa, dst=dst + da, row_bytes=n))
            else:              # pool -> pool, rows of a pitched source packed into the destination
                rb = int(rng.integers(17, 300))
                rows = max(2, n // rb)
                pitch = rb + int(rng.integers(0, 700))
                src, dst = _alloc(engs, rows * pitch + 32, rng), _alloc(engs, rows * rb + 32)
                recs.append(dict(func=f, src_space=FT_POOL, dst_space=FT_POOL, src=src + sa, dst=dst + da, row_bytes=rb,
                                 rows=rows, src_pitch=pitch, dst_pitch=rb))
    return make_descs(recs)


def _images_equal(orc, a, b):
    import torch
    img_a = torch.cat([t for t, _ in a.segments]).cpu().numpy()
    img_b = torch.cat([t for t, _ in b.segments]).cpu().numpy()
    assert np.array_equal(img_b, img_a), "pool image differs from ft_submit_transfers'"
    assert np.array_equal(img_b, orc.pool_mem), "pool image differs from the oracle's"
    n = len(orc.host_mem)
    assert np.array_equal(b.host_np[:n], a.host_np[:n]), "host image differs from ft_submit_transfers'"
    assert np.array_equal(b.host_np[:n], orc.host_mem), "host image differs from the oracle's"


def test_static_submit_twice_matches_the_allocating_submit():
    import torch
    print("case ft_submit_static: 8 functions x 20 pieces, then 2 functions x 3 pieces", flush=True)
    host, pool = 1 << 26, 3 << 27
    orc, a, b, rng = _engines(host, pool, 16384, 2411)
    engs = (orc, a, b)
    try:
        at = [host // 2]
        big = _job(engs, rng, 8, 20, (1000, 900000), at)       # 160 descriptors: ~20 KiB of tables, several pieces
        small = _job(engs, rng, 2, 3, (100, 70000), at)         # fewer functions, fewer bytes, one piece of tables
        w_big, w_small = [1, 1, 2, 2, 4, 4, 8, 8], [3, 1]
        for d, w, C in ((big, w_big, 256 * 1024), (small, w_small, 64 * 1024)):
            orc.wait(orc.submit(d, w, C))
            a.wait(a.submit(d, w, C, fmt.FT_VALIDATE))
        torch.cuda.synchronize()
        # the two static calls back to back, nothing in between
        b.submit_static(big, w_big, 256 * 1024, fmt.FT_VALIDATE)
        b.submit_static(small, w_small, 64 * 1024, fmt.FT_VALIDATE)
        torch.cuda.current_stream().synchronize()
        _images_equal(orc, a, b)
    finally:
        a.close()
        b.close()


def test_static_submit_limits():
    import torch
    from paper_2411_01830_amd import binding as ft
    print("case ft_submit_static: limits", flush=True)
    orc, a, b, rng = _engines(1 << 20, 1 << 24, 4096, 7)
    try:
        src, dst = _alloc((orc, a, b), 1 << 20, rng), _alloc((orc, a, b), 1 << 20)
        many = make_descs([dict(func=i % 4, src_space=FT_POOL, dst_space=FT_POOL, src=src + 512 * i, dst=dst + 512 * i,
                                row_bytes=500) for i in range(2000)])
        before = torch.cat([t for t, _ in b.segments]).cpu().numpy()
        with pytest.raises(ft.FtError) as err:
            b.submit_static(many, [1, 2, 3, 4], 4096)
        assert err.value.code == fmt.FT_E2BIG
        with pytest.raises(ft.FtError) as err:
            b.submit_static(many[:4], [1, 2, 3, 4], 4096, ft.FT_LOG)
        assert err.value.code == fmt.FT_EINVAL
        torch.cuda.synchronize()
        assert np.array_equal(torch.cat([t for t, _ in b.segments]).cpu().numpy(), before)   # nothing was launched
        # what fits is carried out, and an empty submit is valid
        few = many[:600]
        b.submit_static(few, [1, 2, 3, 4], 4096)
        b.submit_static(few[:0], [1], 4096)
        orc.wait(orc.submit(few, [1, 2, 3, 4], 4096))
        a.wait(a.submit(few, [1, 2, 3, 4], 4096))
        torch.cuda.synchronize()
        _images_equal(orc, a, b)
    finally:
        a.close()
        b.close()
