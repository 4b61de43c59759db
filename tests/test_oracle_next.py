"""Pins of the oracle's Sec. 6.1 additions: transfer rate control (SLO -> rates -> integer
weights) and batched triggering with functions that arrive while the link is busy.
None of these tests calls the HIP library."""
import random
from fractions import Fraction

import pytest

from oracle import OracleError
from oracle.batches import batched_order
from oracle.rate import allocate_rates, least_rates, rates_to_weights, slo_weights
from oracle.schedule import stride_order


# ---- rate control ------------------------------------------------------------------

def test_least_rate_is_size_over_transfer_budget():
    # Sec. 6.1: Rate_least = data_size / (L_slo - L_infer). 100 MB, 100 ms SLO, 50 ms of
    # inference leave 50 ms: 2 GB/s. 6 MB in 3 ms: 2 GB/s as well.
    assert least_rates([100e6, 6e6], [0.100, 0.005], [0.050, 0.002]) == pytest.approx([2e9, 2e9], rel=1e-12)


def test_idle_rate_goes_to_the_tightest_slo():
    # 25 GB/s link, least rates 2 and 3 GB/s: 20 GB/s idle, all of it to the function with
    # 10 ms of budget (the other has 50 ms).
    r = allocate_rates([100e6, 30e6], [0.100, 0.020], [0.050, 0.010], 25e9)
    assert r == pytest.approx([2e9, 23e9], rel=1e-12)
    assert sum(r) == pytest.approx(25e9, rel=1e-12)
    # the order of the inputs does not matter, the budget does
    r = allocate_rates([30e6, 100e6], [0.020, 0.100], [0.010, 0.050], 25e9)
    assert r == pytest.approx([23e9, 2e9], rel=1e-12)
    # equal budgets: the lower index takes it
    r = allocate_rates([10e6, 10e6], [0.5, 0.75], [0.25, 0.5], 100e6)   # budgets are 0.25 s exactly
    assert r == pytest.approx([60e6, 40e6], rel=1e-12)


def test_overcommitted_link_adds_nothing():
    r = allocate_rates([100e6, 100e6], [0.02, 0.03], [0.01, 0.01], 12e9)   # needs 10 + 5 GB/s
    assert r == pytest.approx([10e9, 5e9], rel=1e-12)


def test_slo_without_transfer_time_is_an_error():
    for slo, infer in ((0.01, 0.01), (0.01, 0.02)):
        with pytest.raises(OracleError):
            allocate_rates([1e6], [slo], [infer], 1e9)
    with pytest.raises(OracleError):
        allocate_rates([], [], [], 1e9)


def test_weights_are_shares_of_64_rounded_half_up_at_least_one():
    assert rates_to_weights([1.0, 1.0]) == [32, 32]
    assert rates_to_weights([2e9, 23e9]) == [5, 59]          # 5.12 and 58.88
    assert rates_to_weights([1.0, 3.0], total=2) == [1, 2]    # 0.5 rounds up to 1, 1.5 to 2
    assert rates_to_weights([1.0, 1000.0]) == [1, 64]         # never below one
    assert rates_to_weights([5.0]) == [64]


def test_weights_do_not_depend_on_units():
    rng = random.Random(3)
    for _ in range(200):
        n = rng.randint(1, 8)
        size = [rng.randint(1, 1 << 30) for _ in range(n)]
        infer = [rng.uniform(0.001, 0.05) for _ in range(n)]
        slo = [x + rng.uniform(0.001, 0.1) for x in infer]
        bw = rng.uniform(1e9, 64e9)
        w = slo_weights(size, slo, infer, bw)
        assert all(x >= 1 for x in w) and len(w) == n
        assert abs(sum(w) - 64) <= n                          # each entry rounds by at most 1/2, or up to 1
        # bytes and bandwidth in other units (exact power of two: no rounding difference)
        assert slo_weights([s * 1024 for s in size], slo, infer, bw * 1024) == w
        # proportionality: the weights follow the rates within the rounding step
        r = allocate_rates(size, slo, infer, bw)
        for x, y in zip(w, r):
            assert abs(x - max(1.0, y / sum(r) * 64)) <= 0.5 + 1e-9


# ---- batched triggering --------------------------------------------------------------

def _flat(batches):
    return [c for b in batches for c in b]


def _brute_order(funcs, n, w):
    """Every chunk sorted by (finish tag, function position): the definition of the order."""
    keys = []
    for i, _ in enumerate(funcs):
        for k in range(n[i]):
            keys.append((Fraction(k + 1, w[i]), i, k))
    keys.sort()
    return [(i, k) for _, i, k in keys]


def test_no_arrival_is_the_plain_order_cut_in_fives():
    rng = random.Random(5)
    for _ in range(100):
        F = rng.randint(1, 6)
        n = [rng.randint(0, 9) for _ in range(F)]
        w = [rng.choice([1, 2, 3, 4, 8]) for _ in range(F)]
        B = rng.randint(1, 7)
        got = batched_order([{"n": n, "w": w}], B)
        assert _flat(got) == [(0, f, k) for f, k in stride_order(n, w)]
        assert all(len(b) == B for b in got[:-1]) and (not got or 1 <= len(got[-1]) <= B)


def test_hand_derived_merge():
    # tests/golden/batched_orders.txt, case 1
    jobs = [{"n": [6, 6], "w": [1, 1]}, {"n": [2], "w": [4], "arrive": 1}]
    assert batched_order(jobs, 5) == [
        [(0, 0, 0), (0, 1, 0), (0, 0, 1), (0, 1, 1), (0, 0, 2)],
        [(1, 0, 0), (1, 0, 1), (0, 0, 3), (0, 1, 2), (0, 0, 4)],
        [(0, 1, 3), (0, 0, 5), (0, 1, 4), (0, 1, 5)]]
    # case 2: the link ran dry before the second job came
    jobs = [{"n": [3], "w": [1]}, {"n": [2], "w": [1], "arrive": 7}]
    assert batched_order(jobs, 5) == [[(0, 0, 0), (0, 0, 1), (0, 0, 2)], [(1, 0, 0), (1, 0, 1)]]


def test_golden_file_cases():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "batched_orders.txt")
    cases = 0
    with open(path) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if not line:
                continue
            spec, want = line.split("=>")
            B, *js = spec.split("|")
            jobs = []
            for j in js:
                parts = j.split(";")
                job = {"n": [int(x) for x in parts[0].split(",")], "w": [int(x) for x in parts[1].split(",")]}
                if len(parts) > 2:
                    job["arrive"] = int(parts[2])
                jobs.append(job)
            got = " / ".join(" ".join(f"j{a}f{b}c{c}" for a, b, c in batch) for batch in batched_order(jobs, int(B)))
            assert got == want.strip(), line
            cases += 1
    assert cases >= 3


def test_merge_properties_random():
    rng = random.Random(9)
    for case in range(300):
        B = rng.randint(1, 6)
        jobs = []
        njobs = rng.randint(1, 4)
        arrive = sorted(rng.randint(0, 8) for _ in range(njobs - 1))
        for j in range(njobs):
            F = rng.randint(1, 4)
            job = {"n": [rng.randint(0, 8) for _ in range(F)], "w": [rng.choice([1, 1, 2, 3, 5]) for _ in range(F)]}
            if j:
                job["arrive"] = arrive[j - 1]
            jobs.append(job)
        batches = batched_order(jobs, B)
        flat = _flat(batches)
        # every chunk of every function exactly once, each function's chunks in ascending order
        want = sorted((j, f, k) for j, job in enumerate(jobs) for f, n in enumerate(job["n"]) for k in range(n))
        assert sorted(flat) == want, case
        for j, job in enumerate(jobs):
            for f in range(len(job["n"])):
                ks = [k for a, b, k in flat if (a, b) == (j, f)]
                assert ks == sorted(ks)
        assert all(1 <= len(b) <= B for b in batches)
        assert batches == _reference_batches(jobs, B), case


def _reference_batches(jobs, B):
    """The rule written a second way: the remaining work is an explicit list of chunks,
    re-sorted by (finish tag, job, function) whenever jobs join."""
    waiting = list(range(1, len(jobs)))
    present = [0]
    done = {}
    todo = None
    out = []
    while True:
        newly = [j for j in waiting if jobs[j]["arrive"] <= len(out)]
        if todo is not None and not todo and not newly and waiting:
            newly = [waiting[0]]
        if todo is None or newly:
            for j in newly:
                waiting.remove(j)
                present.append(j)
            keys = []
            for j in present:
                for f, n in enumerate(jobs[j]["n"]):
                    have = done.get((j, f), 0)
                    for i in range(n - have):
                        keys.append((Fraction(i + 1, jobs[j]["w"][f]), j, f, have + i))
            keys.sort()
            todo = [(j, f, k) for _, j, f, k in keys]
        if not todo:
            if not waiting:
                return out
            continue
        batch, todo = todo[:B], todo[B:]
        for j, f, _ in batch:
            done[(j, f)] = done.get((j, f), 0) + 1
        out.append(batch)


def test_newcomer_with_high_weight_is_served_within_one_batch_of_arrival():
    # the point of batched triggering: a small urgent function does not wait for the long one
    jobs = [{"n": [1000], "w": [1]}, {"n": [4], "w": [8], "arrive": 10}]
    batches = batched_order(jobs, 5)
    where = [i for i, b in enumerate(batches) for c in b if c[0] == 1]
    assert where == [10, 10, 10, 10]


def _reference_batches_reweighted(jobs, B):
    """The second formulation above with weight changes: the explicit list of remaining chunks is
    re-sorted with the weights then in force whenever jobs join or a change falls due."""
    waiting = list(range(1, len(jobs)))
    present = [0]
    w = [list(j["w"]) for j in jobs]
    changes = [(at, j, list(x)) for j, job in enumerate(jobs) for at, x in job.get("reweight", [])]
    changes.sort(key=lambda t: t[0])
    done = {}
    todo = None
    out = []
    while True:
        newly = [j for j in waiting if jobs[j]["arrive"] <= len(out)]
        if todo is not None and not todo and not newly and waiting:
            newly = [waiting[0]]
        changed = False
        while changes and changes[0][0] <= len(out):
            _, j, x = changes.pop(0)
            w[j] = x
            changed = True
        if todo is None or newly or (changed and todo):
            for j in newly:
                waiting.remove(j)
                present.append(j)
            keys = []
            for j in present:
                for f, n in enumerate(jobs[j]["n"]):
                    have = done.get((j, f), 0)
                    for i in range(n - have):
                        keys.append((Fraction(i + 1, w[j][f]), j, f, have + i))
            keys.sort()
            todo = [(j, f, k) for _, j, f, k in keys]
        if not todo:
            if not waiting:
                return out
            continue
        batch, todo = todo[:B], todo[B:]
        for j, f, _ in batch:
            done[(j, f)] = done.get((j, f), 0) + 1
        out.append(batch)


def test_reweighting_hand_case_and_second_formulation():
    # two functions 1:1, ten chunks each, batches of 4; after two batches function 1 gets weight 3:
    # the first two batches alternate, then of every four chunks three are function 1's until it runs out
    jobs = [{"n": [10, 10], "w": [1, 1], "reweight": [(2, [1, 3])]}]
    got = batched_order(jobs, 4)
    assert got[:2] == [[(0, 0, 0), (0, 1, 0), (0, 0, 1), (0, 1, 1)], [(0, 0, 2), (0, 1, 2), (0, 0, 3), (0, 1, 3)]]
    # tags from the rebuild: f1 at 1/3, 2/3, 1, f0 at 1 (ties to the lower function), ...
    assert got[2] == [(0, 1, 4), (0, 1, 5), (0, 0, 4), (0, 1, 6)]
    assert got[3] == [(0, 1, 7), (0, 1, 8), (0, 0, 5), (0, 1, 9)]
    assert _flat(got[4:]) == [(0, 0, k) for k in range(6, 10)]
    # a change that restores the old weights still restarts the tags (it is a rebuild like any other)
    same = batched_order([{"n": [10, 10], "w": [1, 2], "reweight": [(1, [1, 2])]}], 3)
    assert sorted(_flat(same)) == sorted(_flat(batched_order([{"n": [10, 10], "w": [1, 2]}], 3)))
    # two changes at the same count: the one made later holds
    twice = batched_order([{"n": [10, 10], "w": [1, 1], "reweight": [(2, [5, 1]), (2, [1, 3])]}], 4)
    assert twice == got
    rng = random.Random(13)
    for case in range(300):
        B = rng.randint(1, 6)
        njobs = rng.randint(1, 3)
        arrive = sorted(rng.randint(0, 8) for _ in range(njobs - 1))
        jobs = []
        for j in range(njobs):
            F = rng.randint(1, 3)
            job = {"n": [rng.randint(0, 9) for _ in range(F)], "w": [rng.choice([1, 2, 3, 5]) for _ in range(F)]}
            if j:
                job["arrive"] = arrive[j - 1]
            if rng.random() < 0.7:
                job["reweight"] = sorted(((rng.randint(0, 10), [rng.choice([1, 2, 4, 7]) for _ in range(F)])
                                          for _ in range(rng.randint(1, 2))), key=lambda t: t[0])
            jobs.append(job)
        got = batched_order(jobs, B)
        want = sorted((j, f, k) for j, job in enumerate(jobs) for f, n in enumerate(job["n"]) for k in range(n))
        assert sorted(_flat(got)) == want, case
        assert got == _reference_batches_reweighted(jobs, B), case


def test_rate_rule_drives_the_reweighting():
    """Sec. 6.1 end to end on paper: two functions share the link by their least rates plus the idle
    part for the tighter one; when a third, tighter function arrives the idle part moves to it, so the
    second function's weight drops back to its least rate - the order after the arrival follows the new
    weights of all three."""
    size, slo, infer, bw = [64e6, 64e6], [0.050, 0.020], [0.010, 0.010], 12.8e9
    w2 = slo_weights(size, slo, infer, bw)
    assert w2[1] > w2[0]
    size3, slo3, infer3 = size + [8e6], slo + [0.012], infer + [0.010]
    w3 = slo_weights(size3, slo3, infer3, bw)
    assert w3 == [8, 32, 24] and w2 == [8, 56]       # 1.6, 6.4, 4 GB/s least; 0.8 (then 4.8) GB/s idle moves on
    jobs = [{"n": [40, 40], "w": w2, "reweight": [(3, w3[:2])]}, {"n": [4], "w": [w3[2]], "arrive": 3}]
    got = batched_order(jobs, 5)
    assert got == _reference_batches_reweighted(jobs, 5)
    first_after = [c for b in got[3:5] for c in b]
    assert sum(1 for c in first_after if c[0] == 1) == 4     # the newcomer is through within two batches
