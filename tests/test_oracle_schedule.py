"""Pins for the oracle's chunk order (Sec. 6.1, stride reading)."""
import os
import random
from fractions import Fraction
from math import ceil, floor

import pytest

from oracle import stride_order, chunk_count, chunk_segments

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _golden_orders():
    out = []
    with open(os.path.join(GOLD, "stride_orders.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w, n, order = [x.strip() for x in line.split("|")]
            out.append(([int(x) for x in w.split(",")], [int(x) for x in n.split(",")],
                        [tuple(int(y) for y in x.split(":")) for x in order.split()]))
    return out


@pytest.mark.parametrize("w,n,order", _golden_orders())
def test_hand_derived_orders(w, n, order):
    assert stride_order(n, w) == order


def test_feature_round_golden():
    with open(os.path.join(GOLD, "feature_round.txt")) as fh:
        want = [int(x) for line in fh if not line.startswith("#") for x in line.split()]
    w = [1, 1, 2, 2, 4, 4, 8, 8]
    n = [3 * x for x in w]
    got = stride_order(n, w)
    assert [f for f, _ in got[:30]] == want
    # periodic while everyone is active, and chunk index advances by w_f per round
    assert [f for f, _ in got[30:60]] == want
    seen = {}
    for f, k in got:
        assert k == seen.get(f, 0)
        seen[f] = k + 1


def _random_instance(rng, fmax=6, nmax=12, wmax=9):
    F = rng.randint(1, fmax)
    return [rng.randint(0, nmax) for _ in range(F)], [rng.randint(1, wmax) for _ in range(F)]


def test_matches_sort_by_finish_tag():
    """The order is the sort of every chunk by (finish tag, function)."""
    rng = random.Random(7)
    for _ in range(400):
        n, w = _random_instance(rng)
        brute = sorted(((Fraction(j + 1, w[f]), f, j) for f in range(len(n)) for j in range(n[f])))
        assert stride_order(n, w) == [(f, j) for _, f, j in brute]


def test_closed_form_rank():
    """Ticket of chunk (f, j) = number of chunks sorted before it:
    for g < f those with (i+1)/w_g <= (j+1)/w_f, for g > f those strictly smaller."""
    rng = random.Random(11)
    for _ in range(300):
        n, w = _random_instance(rng)
        order = stride_order(n, w)
        assert sorted(order) == [(f, j) for f in range(len(n)) for j in range(n[f])]
        for t, (f, j) in enumerate(order):
            rank = j
            for g in range(len(n)):
                if g == f:
                    continue
                x = Fraction((j + 1) * w[g], w[f])
                c = floor(x) if g < f else ceil(x) - 1
                rank += min(n[g], c)
            assert rank == t


def test_equal_weights_is_round_robin():
    rng = random.Random(3)
    for _ in range(100):
        F = rng.randint(1, 6)
        n = [rng.randint(0, 9) for _ in range(F)]
        wv = rng.randint(1, 5)
        want = []
        for rnd in range(max(n) if n else 0):
            want += [(f, rnd) for f in range(F) if n[f] > rnd]
        assert stride_order(n, [wv] * F) == want


def test_single_function_in_stream_order():
    assert stride_order([5], [3]) == [(0, k) for k in range(5)]
    assert stride_order([0, 4, 0], [9, 2, 1]) == [(1, k) for k in range(4)]


def test_share_within_one_chunk_at_every_prefix():
    """While functions are active there is a virtual time v with
    v*w_f - 1 <= s_f <= v*w_f for each: max s_f/w_f <= min (s_f+1)/w_f."""
    rng = random.Random(5)
    for _ in range(300):
        n, w = _random_instance(rng, nmax=20)
        s = [0] * len(n)
        for f, k in stride_order(n, w):
            s[f] += 1
            active = [g for g in range(len(n)) if s[g] < n[g]]
            if active:
                assert max(Fraction(s[g], w[g]) for g in active) <= \
                    min(Fraction(s[g] + 1, w[g]) for g in active)


def test_period_and_per_round_counts():
    w = [3, 1, 2, 5]
    W = sum(w)
    n = [4 * x for x in w]
    order = stride_order(n, w)
    first = [f for f, _ in order[:W]]
    for r in range(4):
        assert [f for f, _ in order[r * W:(r + 1) * W]] == first
    for f in range(len(w)):
        assert first.count(f) == w[f]


def test_scaling_all_weights_keeps_the_order():
    rng = random.Random(13)
    for _ in range(100):
        n, w = _random_instance(rng)
        assert stride_order(n, w) == stride_order(n, [3 * x for x in w])


def test_chunk_count():
    assert chunk_count(0, 64) == 0
    assert chunk_count(1, 64) == 1
    assert chunk_count(64, 64) == 1
    assert chunk_count(65, 64) == 2


def test_chunks_cover_every_payload_byte_once():
    rng = random.Random(17)
    for _ in range(200):
        shape = [(rng.randint(1, 40), rng.randint(1, 5)) for _ in range(rng.randint(1, 6))]
        C = 16 * rng.randint(1, 6)
        total = sum(a * b for a, b in shape)
        count = [[0] * (rb * rows) for rb, rows in shape]
        stream_pos = 0
        for k in range(chunk_count(total, C)):
            got = 0
            for d, r, c, length in chunk_segments(shape, C, k):
                rb, rows = shape[d]
                assert 0 <= r < rows and 0 <= c and c + length <= rb and length > 0
                # position in the stream is monotone and contiguous
                base = sum(a * b for a, b in shape[:d])
                assert base + r * rb + c == stream_pos
                stream_pos += length
                got += length
                for i in range(length):
                    count[d][r * rb + c + i] += 1
            assert got == min(C, total - k * C)
        assert all(x == 1 for row in count for x in row)
        assert chunk_segments(shape, C, chunk_count(total, C)) == []
