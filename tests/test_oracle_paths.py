"""Pins of the oracle's path selection (Sec. 6.2, Alg. 1) and chunk striping, and the
library's host-side planner held against it. No GPU."""
import itertools
import random
from fractions import Fraction

import numpy as np
import pytest
from scipy.sparse import csr_matrix
from scipy.sparse.csgraph import maximum_flow

from oracle.paths import Links, dgx_v100_like, edges, simple_paths, stripe_chunks, xgmi_full_mesh
from oracle.schedule import stride_order


def test_simple_paths_against_brute_force_permutations():
    rng = random.Random(1)
    for _ in range(60):
        n = rng.randint(2, 6)
        topo = [[0 if a == b or rng.random() < 0.4 else rng.choice([24, 48]) for b in range(n)] for a in range(n)]
        s, d = rng.sample(range(n), 2)
        hops = rng.choice([0, 1, 2, 3])
        want = []
        others = [v for v in range(n) if v not in (s, d)]
        for k in range(len(others) + 1):
            for mid in itertools.permutations(others, k):
                p = (s,) + mid + (d,)
                if all(topo[u][v] > 0 for u, v in edges(p)) and (hops == 0 or len(p) - 1 <= hops):
                    want.append(p)
        want.sort(key=lambda p: (len(p), p))
        assert simple_paths(topo, s, d, hops) == want


def test_idle_full_mesh_uses_every_link_of_the_source():
    # 8 GPUs, one link between every pair: direct path plus the six two-hop paths = 7 links' worth,
    # which is also the maximum flow.
    L = Links(xgmi_full_mesh(8, 64))
    got = L.select(1, 0, 5)
    assert [p for p, _ in got] == [(0, 5)] + [(0, v, 5) for v in (1, 2, 3, 4, 6, 7)]
    assert sum(bw for _, bw in got) == 7 * 64 == L.total(1)
    assert L.out_free(0) == 0 and L.in_free(5) == 0
    # a second function between two other GPUs still finds its direct link and the relays left
    got = L.select(2, 1, 2)
    assert got[0] == ((1, 2), 64)
    assert all(L.free[u][v] >= 0 for u in range(8) for v in range(8))


def test_hybrid_cube_mesh_by_hand():
    # GPU 0 of the stand-in topology has links to 1, 2 (24 GB/s) and 3, 4 (48 GB/s). 0 -> 3: the direct
    # link (48), then the two-hop paths over 1 and 2 (24 each, their narrowest link), then 0-4-7-3 (48):
    # all 144 GB/s that leave GPU 0.
    L = Links(dgx_v100_like())
    assert L.select(1, 0, 3) == [((0, 3), 48), ((0, 1, 3), 24), ((0, 2, 3), 24), ((0, 4, 7, 3), 48)]
    assert L.out_free(0) == 0
    # nothing leaves GPU 0 any more: a second sender there gets no path, and step 2 does not apply
    assert L.select(2, 0, 1) == []
    L.release(1)
    assert L.free == dgx_v100_like()
    assert [p for p, _ in L.select(3, 0, 1)][:1] == [(0, 1)]


def test_bandwidth_balancing_hand_example():
    # tests/golden/path_balancing.txt: function 2 holds 30 GB/s (3-0 direct, and 3-1-2-0), function 3
    # wants 1 -> 5 and finds only the direct link idle (20); the path 1-2-5 is blocked by function 2's
    # second path alone, function 2 holds more (30 > 20) and can move that path to 3-5-2-0, which shares
    # no link with 1-2-5: it moves, function 3 takes 1-2-5 (10).
    topo = [[0, 0, 10, 20, 0, 0], [0, 0, 20, 10, 20, 20], [10, 20, 0, 0, 0, 10],
            [20, 10, 0, 0, 0, 20], [0, 20, 0, 0, 0, 0], [0, 20, 10, 20, 0, 0]]
    L = Links(topo)
    assert L.select(1, 4, 3) == [((4, 1, 3), 10)]
    assert L.select(2, 3, 0) == [((3, 0), 20), ((3, 1, 2, 0), 10)]
    assert L.select(3, 1, 5) == [((1, 5), 20), ((1, 2, 5), 10)]
    assert [(p, bw) for p, bw in L.paths[2]] == [((3, 0), 20), ((3, 5, 2, 0), 10)]
    assert L.free[1][2] == 10 and L.free[2][0] == 0 and L.free[3][1] == 10


def _check_state(L):
    # what is free plus what the functions hold is the topology; nothing negative
    held = [[0] * L.n for _ in range(L.n)]
    for plist in L.paths.values():
        for p, bw in plist:
            assert bw == min(L.topo[u][v] for u, v in edges(p))
            assert len(set(p)) == len(p)
            for u, v in edges(p):
                held[u][v] += bw
    for u in range(L.n):
        for v in range(L.n):
            assert L.free[u][v] >= 0 and L.free[u][v] + held[u][v] == L.topo[u][v]


def test_random_sequences_keep_the_books_and_respect_max_flow():
    rng = random.Random(13)
    for _ in range(150):
        n = rng.randint(3, 7)
        topo = [[0] * n for _ in range(n)]
        for a in range(n):
            for b in range(a + 1, n):
                if rng.random() < 0.6:
                    topo[a][b] = topo[b][a] = rng.choice([24, 48])
        L = Links(topo, rng.choice([0, 2, 3]))
        nxt = 0
        for _ in range(rng.randint(1, 6)):
            if L.paths and rng.random() < 0.3:
                L.release(rng.choice(list(L.paths)))
            else:
                s, d = rng.sample(range(n), 2)
                nxt += 1
                before_idle = all(L.free[u][v] == topo[u][v] for u in range(n) for v in range(n))
                got = L.select(nxt, s, d)
                # a function's own paths never share a link
                used = [e for p, _ in got for e in edges(p)]
                assert len(used) == len(set(used))
                flow = maximum_flow(csr_matrix(np.array(topo, dtype=np.int32)), s, d).flow_value
                assert sum(bw for _, bw in got) <= flow
                if before_idle and got:
                    assert len(got[0][0]) == len(simple_paths(topo, s, d, L.max_hops)[0])   # a shortest path comes first
            _check_state(L)


def test_striping_is_the_proportional_order_with_paths_as_functions():
    assert stripe_chunks([48, 24, 24], 8) == [0, 0, 1, 2, 0, 0, 1, 2]
    rng = random.Random(2)
    for _ in range(100):
        bw = [rng.choice([24, 48, 64, 10]) for _ in range(rng.randint(1, 5))]
        n = rng.randint(0, 60)
        got = stripe_chunks(bw, n)
        assert got == [f for f, _ in stride_order([n] * len(bw), bw)][:n]
        # at every prefix every path is within one chunk of a common virtual time
        sent = [0] * len(bw)
        for p in got:
            sent[p] += 1
            assert max(Fraction(x, b) for x, b in zip(sent, bw)) <= min(Fraction(x + 1, b) for x, b in zip(sent, bw))


# ---- the library's planner against the oracle ---------------------------------------------------

def test_library_planner_matches_oracle():
    from paper_2411_01830_amd import binding as ft
    rng = random.Random(17)
    for case in range(120):
        if case == 0:
            topo, hops = dgx_v100_like(), 0
        elif case == 1:
            topo, hops = xgmi_full_mesh(8, 64), 3
        else:
            n = rng.randint(2, 7)
            topo = [[0] * n for _ in range(n)]
            for a in range(n):
                for b in range(n):
                    if a != b and rng.random() < 0.6:
                        topo[a][b] = rng.choice([24, 48])
            hops = rng.choice([0, 2, 3])
        n = len(topo)
        lib, orc = ft.Links(topo, hops), Links(topo, hops)
        nxt = 0
        for _ in range(rng.randint(1, 8)):
            if orc.paths and rng.random() < 0.3:
                g = rng.choice(list(orc.paths))
                orc.release(g)
                lib.release(g)
            else:
                s, d = rng.sample(range(n), 2)
                nxt += 1
                assert lib.select(nxt, s, d) == orc.select(nxt, s, d)
            assert lib.free() == orc.free
            for g, plist in orc.paths.items():
                assert lib.paths(g) == [(p, bw) for p, bw in plist]
        lib.close()
    for _ in range(200):
        bw = [rng.choice([24, 48, 64, 10, 7]) for _ in range(rng.randint(1, 6))]
        n = rng.randint(0, 100)
        assert ft.stripe_chunks(bw, n) == stripe_chunks(bw, n)
    with pytest.raises(ft.FtError):
        ft.Links([[0, 1], [1, 0]]).select(1, 0, 0)
