"""Pins for the oracle's slab pool (Sec. 7.1; first-fit reading)."""
import random

import pytest

from oracle import Pool, OracleError, EINVAL, ENOMEM


def _brute_first_fit(bitmap, seg_bounds, need):
    """Reference model: try every start index in increasing order."""
    for start in range(len(bitmap)):
        end = start + need
        if end > len(bitmap):
            break
        if any((start < b < end) for b in seg_bounds):     # run would straddle a segment edge
            continue
        if all(not bitmap[i] for i in range(start, end)):
            return start
    return None


def test_random_alloc_free_against_bitmap_model():
    rng = random.Random(1)
    for trial in range(30):
        slab = 256 * rng.randint(1, 4)
        nseg = [rng.randint(3, 24)]
        pool = Pool(nseg[0] * slab, slab)
        bitmap = [False] * nseg[0]
        live = {}
        for step in range(200):
            r = rng.random()
            if r < 0.05 and len(bitmap) < 64:
                add = rng.randint(1, 16)
                pool.grow(add * slab)
                nseg.append(add)
                bitmap += [False] * add
            elif r < 0.6 or not live:
                nbytes = rng.randint(1, 6 * slab)
                need = -(-nbytes // slab)
                bounds = []
                acc = 0
                for x in nseg[:-1]:
                    acc += x
                    bounds.append(acc)
                want = _brute_first_fit(bitmap, bounds, need)
                if want is None:
                    with pytest.raises(OracleError) as ei:
                        pool.alloc(nbytes)
                    assert ei.value.code == ENOMEM
                else:
                    off = pool.alloc(nbytes)
                    assert off == want * slab
                    for i in range(want, want + need):
                        assert not bitmap[i]
                        bitmap[i] = True
                    live[off] = need
            else:
                off = rng.choice(list(live))
                need = live.pop(off)
                pool.free(off)
                for i in range(off // slab, off // slab + need):
                    bitmap[i] = False
            # live allocations never overlap and are slab aligned
            spans = sorted((o, o + n * slab) for o, n in live.items())
            for (a0, a1), (b0, b1) in zip(spans, spans[1:]):
                assert a1 <= b0
            assert all(o % slab == 0 for o in live)


def test_free_then_alloc_same_size_returns_same_offset():
    pool = Pool(16 * 4096, 4096)
    a = pool.alloc(5000)
    b = pool.alloc(100)
    c = pool.alloc(3 * 4096)
    assert (a, b, c) == (0, 2 * 4096, 3 * 4096)
    pool.free(b)
    assert pool.alloc(4096) == b
    pool.free(a)
    assert pool.alloc(2 * 4096) == a


def test_full_pool_then_grow():
    pool = Pool(4 * 1024, 1024)
    pool.alloc(4 * 1024)
    with pytest.raises(OracleError) as ei:
        pool.alloc(1)
    assert ei.value.code == ENOMEM
    pool.grow(2 * 1024)
    assert pool.alloc(1) == 4 * 1024


def test_allocation_never_straddles_segments():
    pool = Pool(4 * 1024, 1024)
    pool.grow(4 * 1024)
    pool.alloc(3 * 1024)            # slabs 0..2; slab 3 free, segment 2 free
    assert pool.alloc(2 * 1024) == 4 * 1024     # not 3*1024: would cross the edge
    assert pool.alloc(1024) == 3 * 1024


def test_bad_arguments():
    for args in ((0, 1024), (1024, 0), (1000, 1024), (1024, 100), (1024 * 3, 512 + 128)):
        with pytest.raises(OracleError) as ei:
            Pool(*args)
        assert ei.value.code == EINVAL
    pool = Pool(4096, 1024)
    for bad in (0, -5):
        with pytest.raises(OracleError) as ei:
            pool.alloc(bad)
        assert ei.value.code == EINVAL
    with pytest.raises(OracleError) as ei:
        pool.grow(100)
    assert ei.value.code == EINVAL
    a = pool.alloc(10)
    with pytest.raises(OracleError) as ei:
        pool.free(a + 1024)
    assert ei.value.code == EINVAL
    pool.free(a)
    with pytest.raises(OracleError) as ei:
        pool.free(a)                # double free
    assert ei.value.code == EINVAL
