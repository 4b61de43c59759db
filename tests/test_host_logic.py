"""The library's host side, without a GPU: exports, pool, schedule tables, validation.

The expected values come from the oracle; the library is called through its C ABI.
No call here reaches the device (every submit either fails validation or is empty)."""
import ctypes
import os
import random
import re

import numpy as np
import pytest

import oracle
from oracle import OracleEngine, OracleError, stride_order
from paper_2411_01830_amd import binding as ft
from workloads import make_descs, FT_HOST, FT_POOL
from workloads import format as fmt

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_BASE = 0x7F0000000000          # never dereferenced: no descriptor passes validation here


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "faastube.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(ft_[a-z_0-9]+)\s*\(", text))
    assert {"ft_pool_create", "ft_slab_alloc", "ft_slab_free", "ft_pool_grow",
            "ft_submit_transfers", "ft_wait"} <= declared
    lib = ctypes.CDLL(ft.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(ft.EXPORTS)


def test_constants_match_between_header_binding_and_shared_format():
    text = open(os.path.join(ROOT, "include", "faastube.h")).read()
    for name in ("FT_EINVAL", "FT_ENOMEM", "FT_ERANGE", "FT_EOVERLAP", "FT_EBUSY", "FT_EHIP"):
        m = re.search(name + r"\s*=\s*(-?\d+)", text)
        assert int(m.group(1)) == getattr(fmt, name)
    for name in ("FT_VALIDATE", "FT_LOG", "FT_PATH_DMA", "FT_TIMING", "FT_DETACHED"):
        m = re.search(name + r"\s*=\s*1\s*<<\s*(\d+)", text)
        assert 1 << int(m.group(1)) == getattr(fmt, name) == getattr(ft, name)
    assert (oracle.EINVAL, oracle.ENOMEM, oracle.ERANGE, oracle.EOVERLAP, oracle.EBUSY) == \
        (fmt.FT_EINVAL, fmt.FT_ENOMEM, fmt.FT_ERANGE, fmt.FT_EOVERLAP, fmt.FT_EBUSY)
    assert ctypes.sizeof(ft.JobStats) == 3 * 56 + 8


def test_header_is_plain_c_and_its_layouts_are_the_bindings(tmp_path):
    """The public header must compile as C99 on its own, and the structures it declares must have the
    sizes and field offsets that the Python side marshals (the descriptor record, the stats records)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    fields = [n for n in fmt.DESC_DTYPE.names]
    src = ['#include <stddef.h>', '#include <stdio.h>', '#include "faastube.h"', 'int main(void) {',
           '  printf("%zu %zu %zu\\n", sizeof(ft_desc), sizeof(ft_class_stats), sizeof(ft_job_stats_t));']
    for n in fields:
        src.append(f'  printf("{n} %zu\\n", offsetof(ft_desc, {n}));')
    for n, _ in ft.ClassStats._fields_:
        src.append(f'  printf("{n} %zu\\n", offsetof(ft_class_stats, {n}));')
    src += ['  printf("%d %d %d %d %d\\n", FT_HOST, FT_POOL, FT_PAGEABLE, FT_OPEN, FT_ECLOSED);', '  return 0;', '}']
    c = tmp_path / "layout.c"
    c.write_text("\n".join(src))
    exe = tmp_path / "layout"
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    str(c), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    assert out[0].split() == ["64", str(ctypes.sizeof(ft.ClassStats)), str(ctypes.sizeof(ft.JobStats))]
    got = dict(line.split() for line in out[1:1 + len(fields)])
    assert {n: int(v) for n, v in got.items()} == {n: fmt.DESC_DTYPE.fields[n][1] for n in fields}
    got = dict(line.split() for line in out[1 + len(fields):1 + len(fields) + len(ft.ClassStats._fields_)])
    assert {n: int(v) for n, v in got.items()} == {n: getattr(ft.ClassStats, n).offset for n, _ in ft.ClassStats._fields_}
    assert [int(v) for v in out[-2].split()] == [FT_HOST, FT_POOL, oracle.PAGEABLE, ft.FT_OPEN, ft.FT_ECLOSED]


def _both(op, lib_call, oracle_call):
    """Run the same call on both; return ('ok', value) or ('err', code) for each."""
    def run(fn):
        try:
            return ("ok", fn())
        except (ft.FtError, OracleError) as e:
            return ("err", e.code)
    a, b = run(lib_call), run(oracle_call)
    assert a == b, (op, a, b)
    return a


def test_pool_matches_oracle_on_random_sequences():
    rng = random.Random(2)
    for trial in range(25):
        slab = 256 * rng.randint(1, 8)
        n0 = rng.randint(2, 40)
        pool = ft.pool_create(FAKE_BASE, n0 * slab, slab, 0)
        orc = oracle.Pool(n0 * slab, slab)
        live = []
        next_base = FAKE_BASE + (1 << 32)
        for step in range(300):
            r = rng.random()
            if r < 0.04:
                add = rng.randint(1, 20) * slab
                _both("grow", lambda: ft.pool_grow(pool, next_base, add), lambda: orc.grow(add))
                next_base += 1 << 32
            elif r < 0.6 or not live:
                nbytes = rng.randint(1, 7 * slab)
                res = _both("alloc", lambda: ft.slab_alloc(pool, nbytes), lambda: orc.alloc(nbytes))
                if res[0] == "ok":
                    live.append(res[1])
            else:
                off = live.pop(rng.randrange(len(live)))
                _both("free", lambda: ft.slab_free(pool, off), lambda: orc.free(off))
        _both("free-bad", lambda: ft.slab_free(pool, 12345 * slab), lambda: orc.free(12345 * slab))
        ft.pool_destroy(pool)


def test_pool_ptr_follows_segments():
    slab = 1024
    pool = ft.pool_create(FAKE_BASE, 4 * slab, slab, 0)
    ft.pool_grow(pool, FAKE_BASE + (1 << 30), 2 * slab)
    assert ft.pool_ptr(pool, 0) == FAKE_BASE
    assert ft.pool_ptr(pool, 4 * slab - 1) == FAKE_BASE + 4 * slab - 1
    assert ft.pool_ptr(pool, 4 * slab + 5) == FAKE_BASE + (1 << 30) + 5
    assert ft.pool_ptr(pool, 6 * slab) is None
    ft.pool_destroy(pool)


def test_pool_create_argument_rules():
    for base, nbytes, slab in ((0, 1024, 256), (FAKE_BASE, 0, 256), (FAKE_BASE, 1000, 256),
                               (FAKE_BASE, 1024, 0), (FAKE_BASE, 1024, 100), (FAKE_BASE + 16, 1024, 256)):
        with pytest.raises(ft.FtError) as ei:
            ft.pool_create(base, nbytes, slab, 0)
        assert ei.value.code == fmt.FT_EINVAL
    pool = ft.pool_create(FAKE_BASE, 1024, 256, 0)
    for base, nbytes in ((0, 256), (FAKE_BASE + 8, 256), (FAKE_BASE, 100)):
        with pytest.raises(ft.FtError) as ei:
            ft.pool_grow(pool, base, nbytes)
        assert ei.value.code == fmt.FT_EINVAL
    with pytest.raises(ft.FtError) as ei:
        ft.slab_alloc(pool, 0)
    assert ei.value.code == fmt.FT_EINVAL
    ft.pool_destroy(pool)


def test_slab_alloc_is_microseconds():
    import time
    slab = 1 << 20
    pool = ft.pool_create(FAKE_BASE, 16384 * slab, slab, 0)
    t0 = time.perf_counter()
    offs = [ft.slab_alloc(pool, (i % 7 + 1) * slab) for i in range(3000)]
    for o in offs[::2]:
        ft.slab_free(pool, o)
    for i in range(1500):
        ft.slab_alloc(pool, (i % 3 + 1) * slab)
    per_call = (time.perf_counter() - t0) / 6000
    ft.pool_destroy(pool)
    assert per_call < 200e-6        # native allocation is millisecond-level (Sec. 7.1)


def test_schedule_tables_match_oracle_order():
    rng = random.Random(4)
    for _ in range(400):
        F = rng.randint(1, 8)
        C = 16 * rng.randint(1, 8)
        n = [rng.randint(0, 25) for _ in range(F)]
        w = [rng.choice([1, 1, 2, 3, 4, 6, 8, 9, 30]) for _ in range(F)]
        S = [0 if x == 0 else x * C - rng.randint(0, C - 1) for x in n]
        assert ft.plan_schedule(S, w, C) == stride_order(n, w)


def test_tickets_name_every_nonempty_tile_once_in_chunk_order():
    """Tickets skip the empty tiles past the end of each function's last chunk: the list
    must be the oracle's chunk order with every chunk cut into tiles, nothing else."""
    rng = random.Random(11)
    for case in range(300):
        F = rng.randint(1, 8)
        C = 16 * rng.randint(1, 64)
        want_tile = 16 * rng.randint(1, 24)
        n = [rng.randint(0, 12) for _ in range(F)]
        w = [rng.choice([1, 1, 2, 3, 4, 8]) for _ in range(F)]
        S = [0 if x == 0 else x * C - rng.randint(0, C - 1) for x in n]
        got = ft.plan_tickets(S, w, C, want_tile)
        # the planner's tile shape: equal tiles, multiple of 16, at most `want_tile` rounded
        ntile = -(-C // max(want_tile, 16))
        tile = -(-(-(-C // ntile)) // 16) * 16
        expect = []
        for f, k in stride_order(n, w):
            lo, hi = k * C, min((k + 1) * C, S[f])
            b = lo
            while b < hi:
                expect.append((f, k, b, min(tile, lo + C - b, hi - b)))
                b += tile
        assert got == expect, (case, S, w, C, want_tile)
        assert all(x[3] > 0 for x in got)
        assert sum(x[3] for x in got) == sum(S)


def test_schedule_tables_weights_dwarf_chunk_counts():
    # weights far larger than the number of chunks: only irregular rounds exist
    w = [1000, 999, 7]
    n = [3, 5, 2]
    assert ft.plan_schedule([x * 64 for x in n], w, 64) == stride_order(n, w)
    # common factor in the weights is divided out
    assert ft.plan_schedule([640, 1280], [1 << 30, 1 << 31], 64) == stride_order([10, 20], [1, 2])


def test_schedule_config_sizes():
    w = [1, 1, 2, 2, 4, 4, 8, 8]
    n = [40, 41, 80, 79, 150, 161, 333, 300]
    assert ft.plan_schedule([x * 2097152 for x in n], w, 2097152) == stride_order(n, w)


def test_schedule_rejects_oversized_slot_tables():
    with pytest.raises(ft.FtError) as ei:
        ft.plan_schedule([64 * (1 << 23)] * 2, [(1 << 23) - 1, (1 << 23) - 3], 64)
    assert ei.value.code == fmt.FT_EINVAL


def _setup_pair():
    slab = 1024
    pool = ft.pool_create(FAKE_BASE, 64 * slab, slab, 0)
    host_base = 0x7E0000000000
    ft.host_window_add(pool, host_base, 1 << 16)
    orc = OracleEngine()
    orc.host_arena(1 << 16)
    orc.pool_create(64 * slab, slab)
    return pool, orc, host_base


def _submit_both(pool, orc, host_base, recs, w, C, flags=fmt.FT_VALIDATE):
    d = make_descs(recs)
    dl = d.copy()
    dl["src"][dl["src_space"] == FT_HOST] += np.uint64(host_base)
    dl["dst"][dl["dst_space"] == FT_HOST] += np.uint64(host_base)
    return _both("submit", lambda: ft.submit_transfers(pool, dl, w, C, flags),
                 lambda: orc.submit(d, w, C))


def test_submit_validation_matches_oracle():
    pool, orc, hb = _setup_pair()
    a = _both("alloc", lambda: ft.slab_alloc(pool, 2048), lambda: orc.slab_alloc(2048))[1]
    good = dict(func=0, src_space=FT_HOST, dst_space=FT_POOL, src=0, dst=a, row_bytes=100)
    E = fmt
    cases = [
        ([good], [0], 64, E.FT_EINVAL),
        ([good], [1], 0, E.FT_EINVAL),
        ([good], [1], 24, E.FT_EINVAL),
        ([dict(good, func=1)], [1], 64, E.FT_EINVAL),
        ([dict(good, flags=1)], [1], 64, E.FT_EINVAL),
        ([dict(good, dst_space=FT_HOST)], [1], 64, E.FT_EINVAL),
        ([dict(good, src_space=3)], [1], 64, E.FT_EINVAL),
        ([dict(good, dst_space=3)], [1], 64, E.FT_EINVAL),
        # ordinary host memory is a host side like the pinned one: never both sides
        ([dict(good, dst_space=2)], [1], 64, E.FT_EINVAL),
        ([dict(good, src_space=2, dst_space=FT_HOST)], [1], 64, E.FT_EINVAL),
        ([dict(good, src_space=2, dst_space=2)], [1], 64, E.FT_EINVAL),
        # ... and with no window declared for it every range in it is outside
        ([dict(good, src_space=2)], [1], 64, E.FT_ERANGE),
        ([dict(good, src_space=FT_POOL, src=a, dst_space=2, dst=64)], [1], 64, E.FT_ERANGE),
        ([dict(good, row_bytes=0)], [1], 64, E.FT_EINVAL),
        ([dict(good, rows=0)], [1], 64, E.FT_EINVAL),
        ([dict(good, rows=2, src_pitch=99, dst_pitch=100)], [1], 64, E.FT_EINVAL),
        ([dict(good, rows=2, src_pitch=100, dst_pitch=99)], [1], 64, E.FT_EINVAL),
        ([dict(good, dst=a + 2048 - 99)], [1], 64, E.FT_ERANGE),
        ([dict(good, dst=a + 4096)], [1], 64, E.FT_ERANGE),
        ([dict(good, rows=3, src_pitch=100, dst_pitch=1000)], [1], 64, E.FT_ERANGE),
        ([dict(good, src=(1 << 16) - 50)], [1], 64, E.FT_ERANGE),
        ([dict(good, rows=1 << 40, row_bytes=1 << 30, src_pitch=1 << 30, dst_pitch=1 << 30)], [1], 64, E.FT_ERANGE),
        ([good, dict(good, src=200, dst=a + 99)], [1], 64, E.FT_EOVERLAP),
        ([dict(good, src_space=FT_POOL, src=a + 50)], [1], 64, E.FT_EOVERLAP),
        ([dict(good, src_space=FT_POOL, src=a + 895, rows=4, row_bytes=10, src_pitch=10, dst_pitch=300)],
         [1], 64, E.FT_EOVERLAP),
        ([dict(good, dst=a + 4096), dict(good, row_bytes=0)], [1], 64, E.FT_EINVAL),
        ([good, dict(good, src=200, dst=a + 99), dict(good, dst=a + 4096)], [1], 64, E.FT_ERANGE),
    ]
    for recs, w, C, want in cases:
        got = _submit_both(pool, orc, hb, recs, w, C)
        assert got == ("err", want), (recs, got)
    # an empty submit is valid on both and completes at once
    res = _submit_both(pool, orc, hb, [], [1], 64)
    assert res[0] == "ok"
    ft.wait(pool, res[1])
    with pytest.raises(ft.FtError) as ei:
        ft.wait(pool, res[1])
    assert ei.value.code == E.FT_EINVAL
    # null descriptor pointer with a non-zero count, and no functions at all
    lib = ctypes.CDLL(ft.LIB_PATH)
    job = ctypes.c_uint64()
    w1 = (ctypes.c_uint32 * 1)(1)
    lib.ft_submit_transfers.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint32, ctypes.c_void_p,
                                        ctypes.c_uint32, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p,
                                        ctypes.POINTER(ctypes.c_uint64)]
    assert lib.ft_submit_transfers(pool, None, 3, w1, 1, 64, 0, None, ctypes.byref(job)) == E.FT_EINVAL
    assert lib.ft_submit_transfers(pool, None, 0, w1, 0, 64, 0, None, ctypes.byref(job)) == E.FT_EINVAL
    ft.pool_destroy(pool)


def test_random_overlap_decisions_match_oracle():
    """Random small batches inside one allocation: both sides agree on accept/reject.
    Accepted batches would need the device, so only rejected ones are submitted to the
    library; the accepted ones are checked through the oracle's brute-force pin instead."""
    pool, orc, hb = _setup_pair()
    a = _both("alloc", lambda: ft.slab_alloc(pool, 8192), lambda: orc.slab_alloc(8192))[1]
    rng = random.Random(8)
    rejected = 0
    for _ in range(400):
        recs = []
        for _ in range(rng.randint(2, 4)):
            rows = rng.choice([1, 2, 3])
            rb = rng.randint(1, 40)
            recs.append(dict(func=0, src_space=rng.choice([FT_HOST, FT_POOL]), dst_space=FT_POOL,
                             src=a + rng.randint(0, 300), dst=a + rng.randint(0, 300), row_bytes=rb,
                             rows=rows, src_pitch=rb + rng.randint(0, 9), dst_pitch=rb + rng.randint(0, 9)))
        for r in recs:
            if r["src_space"] == FT_HOST:
                r["src"] -= a
        d = make_descs(recs)
        if oracle.engine.find_overlap(d):
            rejected += 1
            assert _submit_both(pool, orc, hb, recs, [1], 64) == ("err", fmt.FT_EOVERLAP)
    assert rejected > 100
    ft.pool_destroy(pool)


def test_slo_weights_match_the_oracle_rule():
    """Sec. 6.1 transfer rate control: the library's host routine and the oracle compute the
    same expression in the same order in IEEE double, so rates and weights are identical."""
    from oracle.rate import allocate_rates, slo_weights
    rng = random.Random(21)
    for _ in range(500):
        n = rng.randint(1, 10)
        size = [rng.randint(0, 1 << 31) for _ in range(n)]
        infer = [rng.uniform(0.0005, 0.05) for _ in range(n)]
        slo = [x + rng.uniform(0.0005, 0.2) for x in infer]
        bw = rng.uniform(1e8, 64e9)
        total = rng.choice([0, 16, 64, 1000])
        rates, weights = ft.slo_weights(size, slo, infer, bw, total)
        assert rates == allocate_rates(size, slo, infer, bw)
        assert weights == slo_weights(size, slo, infer, bw, total or 64)
    for bad in (([1.0], [0.01], [0.01], 1e9), ([1.0], [0.01], [0.02], 1e9), ([1.0], [0.02], [0.01], 0.0)):
        with pytest.raises(ft.FtError) as ei:
            ft.slo_weights(*bad)
        assert ei.value.code == fmt.FT_EINVAL


_OBJECTS = {}   # (compiler flags, source) -> object file, shared by the tests of one session


def _build_for_host(tmp_path, exe, flags, sources):
    """Compile the sources (in parallel, each once per set of flags) and link them; returns the compiler's result."""
    import subprocess
    import tempfile
    from concurrent.futures import ThreadPoolExecutor
    cache = _OBJECTS.setdefault("dir", tempfile.mkdtemp(prefix="ft_host_objects_"))

    def compile_one(src):
        key = (tuple(flags), src)
        if key not in _OBJECTS:
            obj = os.path.join(cache, "%d_%s.o" % (abs(hash(key)) % 10 ** 9, os.path.basename(src)))
            res = subprocess.run([*flags, "-c", src, "-o", obj], capture_output=True, text=True)
            if res.returncode != 0:
                return res
            _OBJECTS[key] = obj
        return None
    with ThreadPoolExecutor(max_workers=4) as pool:
        for res in pool.map(compile_one, sources):
            if res is not None:
                return res
    return subprocess.run([*flags, *[_OBJECTS[(tuple(flags), src)] for src in sources], "-o", exe], capture_output=True, text=True)


def _host_sanitizer_run(tmp_path, name, sources, args, expect, sanitize="address,undefined", extra=(), extra_sources=(), env=None):
    """Build tests/host/<name>.cpp with the given library sources for the host, with sanitizers, and run it."""
    import shutil
    import subprocess
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no host compiler")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    csrc = os.path.join(root, "paper_2411_01830_amd", "csrc")
    exe = str(tmp_path / name)
    flags = [gxx, "-std=c++17", "-O1", "-g", "-fsanitize=" + sanitize, "-fno-sanitize-recover=undefined", "-pthread", *extra]
    files = [os.path.join(root, "tests", "host", name + ".cpp"), *extra_sources, *[os.path.join(csrc, f) for f in sources]]
    res = _build_for_host(tmp_path, exe, flags, files)
    plain = [c for c in flags if "sanitize" not in c]
    if res.returncode != 0 and "sanitize" in res.stderr:
        res = _build_for_host(tmp_path, exe, plain, files)
    assert res.returncode == 0, res.stderr[-2000:]
    env = dict(os.environ, **(env or {}))
    run = subprocess.run([exe, *args], capture_output=True, text=True, timeout=300, env=env)
    if run.returncode != 0 and "runtime does not come first" in run.stderr:
        # another library is preloaded ahead of the sanitizer's: run the program's own checks alone
        res = _build_for_host(tmp_path, exe, plain, files)
        assert res.returncode == 0, res.stderr[-2000:]
        run = subprocess.run([exe, *args], capture_output=True, text=True, timeout=300)
    if run.returncode != 0 and "unexpected memory mapping" in run.stderr:
        pytest.skip("the thread sanitizer cannot run under this kernel's address space layout")
    assert run.returncode == 0, (run.stdout[-1000:], run.stderr[-3000:])
    assert expect in run.stdout


def test_every_ticket_walks_the_tables_in_bounds(tmp_path):
    """tests/host/walk_tables.cpp: the planner's sources compiled for the host with sanitizers, random
    submits, every ticket decoded as the kernel decodes it with each table read bounds-checked."""
    _host_sanitizer_run(tmp_path, "walk_tables", ["ft_plan.cpp", "ft_pool.cpp"], ["1", "150"], "done 1..150")


def test_policy_and_path_planners_under_sanitizers(tmp_path):
    """tests/host/policy_calls.cpp: random calls of the migration planner, the pool sizer, the path planner
    and the striping with output arrays of exactly the promised size (leaks included)."""
    _host_sanitizer_run(tmp_path, "policy_calls", ["ft_policy.cpp", "ft_paths.cpp"], ["1", "300"], "done 1..300")


def test_every_code_has_a_name_and_a_fresh_pool_no_hip_error():
    codes = [fmt.FT_OK, fmt.FT_EINVAL, fmt.FT_ENOMEM, fmt.FT_ERANGE, fmt.FT_EOVERLAP, fmt.FT_EBUSY, fmt.FT_EHIP,
             fmt.FT_ECLOSED, fmt.FT_E2BIG]
    names = [ft.strerror(c) for c in codes]
    assert all(names) and len(set(names)) == len(names)
    assert ft.strerror(-99) and ft.strerror(-99) not in names        # an unknown code still gets a text
    # a pool handle needs no GPU (no HIP call before the first submit): its error text starts empty
    pool = ft.pool_create(1 << 20, 1 << 20, 4096, 0)
    assert ft._lib.ft_last_hip_error(pool) == b""
    with pytest.raises(ft.FtError) as err:
        ft.slab_alloc(pool, 2 << 20)
    assert err.value.code == fmt.FT_ENOMEM and ft.strerror(fmt.FT_ENOMEM) in str(err.value)
    ft.pool_destroy(pool)


HOST_SOURCES = ["ft_pool.cpp", "ft_plan.cpp", "ft_api.cpp", "ft_open.cpp", "ft_policy.cpp", "ft_store.cpp", "ft_paths.cpp"]


def _with_the_stand_in(tmp_path, sanitize, rounds, program="c_abi_stress", args=None, expect="c_abi_stress done"):
    """tests/host/c_abi_stress.cpp over the library's host sources, with tests/host/hip_stand_in.cpp in place of
    the HIP runtime and of the kernels (test infrastructure: the library itself has no CPU path)."""
    rocm = "/opt/rocm/include"
    if not os.path.exists(os.path.join(rocm, "hip", "hip_runtime_api.h")):
        pytest.skip("no HIP headers")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    _host_sanitizer_run(tmp_path, program, HOST_SOURCES, [str(rounds), "16"] if args is None else args, expect, sanitize=sanitize,
                        extra=["-D__HIP_PLATFORM_AMD__", "-I" + rocm, "-w"],
                        extra_sources=[os.path.join(root, "tests", "host", "hip_stand_in.cpp")],
                        # streams, events, table buffers and parked threads are kept for the life of the process
                        env={"ASAN_OPTIONS": "detect_leaks=0"})


def test_host_threads_race_free_under_the_thread_sanitizer(tmp_path):
    """An open job that two threads merge into while a third changes its weights and the main thread waits,
    closed jobs on all launch routes, the store: every byte compared with memcpy's, no data race reported."""
    _with_the_stand_in(tmp_path, "thread", 6)


def test_host_code_clean_under_address_and_ub_sanitizers(tmp_path):
    _with_the_stand_in(tmp_path, "address,undefined", 6)


def test_error_paths_with_injected_runtime_failures(tmp_path):
    """tests/host/fault_paths.cpp: the n-th call of each runtime function (and of the kernel launch) fails in turn
    while closed jobs, an open job, a merge and a weight change are attempted. Every call returns a code, nothing
    hangs or stays busy, and the same jobs succeed byte for byte afterwards."""
    _with_the_stand_in(tmp_path, "address,undefined", 0, program="fault_paths", args=[], expect="fault_paths done")


def test_rest_of_the_api_under_sanitizers(tmp_path):
    """tests/host/api_tour.cpp: logs with exactly-sized arrays, the device's order against the host planner's, the
    piece-by-piece comparison path, tuned launch shapes, pitched pieces in all classes, pool growth and shrinkage."""
    _with_the_stand_in(tmp_path, "address,undefined", 0, program="api_tour", args=[], expect="api_tour done")


def test_bench_traffic_constants_are_the_figures_in_the_profiles():
    """bench.py cannot read hardware counters inside the run it times: `roofline.traffic` comes from constants taken
    from rocprofv3 counter runs of the same command. Each constant must be the figure its summary under profiles/
    states (`traffic / algorithmic = X`), so that a refreshed profile and a stale constant cannot go unnoticed."""
    import ast
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    tree = ast.parse(open(os.path.join(root, "bench.py")).read())
    table = None
    for node in tree.body:
        if isinstance(node, ast.Assign) and getattr(node.targets[0], "id", "") == "TRAFFIC_PER_ALGO_BYTE":
            table = ast.literal_eval(node.value)
    assert table and set(table) == {"large_mixed", "feature", "traffic_crops"}
    for name, (factor, path) in table.items():
        text = open(os.path.join(root, path)).read()
        found = re.findall(r"traffic / algorithmic = ([0-9.]+[0-9])", text)
        assert found, f"{path} states no `traffic / algorithmic = X`"
        assert float(found[-1]) == factor, (name, factor, found)
        assert "bench.py" in text and "rocprofv3 --pmc" in text
