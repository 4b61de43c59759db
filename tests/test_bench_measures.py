"""The statistics bench.py derives from the copy kernel's log, checked without a GPU on orders the oracle produces:
the timed-share error of Sec. 6.1's proportional triggering, the distance from the fluid weighted share, and the
union of busy intervals that the pool->pool roofline divides by."""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import bench  # noqa: E402  (imports no GPU code at module level)
from oracle.schedule import stride_order  # noqa: E402


def _tickets(stream_bytes, weights, chunk):
    n = [-(-s // chunk) for s in stream_bytes]
    order = stride_order(n, weights)
    func = np.array([f for f, _ in order], dtype=np.int64)
    nbytes = np.array([min(chunk, stream_bytes[f] - k * chunk) for f, k in order], dtype=np.int64)
    return func, nbytes


def test_fluid_lag_of_the_stride_order_stays_within_two_chunks():
    rng = np.random.default_rng(5)
    for _ in range(30):
        F = int(rng.integers(1, 9))
        w = [int(x) for x in rng.choice([1, 2, 3, 4, 8], F)]
        S = [int(x) for x in rng.integers(1, 60000, F)]
        func, nbytes = _tickets(S, w, 1000)
        worst, p99 = bench.fluid_lag(func, nbytes, w, 1000, np.arange(len(func)))
        assert worst < 2.0 and p99 <= worst, (S, w, worst)


def test_fluid_lag_of_one_function_is_zero_and_of_a_wrong_order_is_large():
    func, nbytes = _tickets([50000], [3], 1000)
    assert bench.fluid_lag(func, nbytes, [3], 1000, np.arange(len(func)))[0] == 0.0
    # two equal functions served one after the other instead of in turn: the second lags by half its stream
    func = np.array([0] * 40 + [1] * 40)
    nbytes = np.full(80, 1000)
    worst, _ = bench.fluid_lag(func, nbytes, [1, 1], 1000, np.arange(80))
    assert 19.5 <= worst <= 20.5
    # the same tickets completing in proportional order (as times would say) are back within a chunk
    order = np.argsort(np.concatenate([np.arange(40) * 2, np.arange(40) * 2 + 1]), kind="stable")
    assert bench.fluid_lag(func, nbytes, [1, 1], 1000, order)[0] <= 0.5


def test_fluid_lag_hands_a_finished_functions_share_to_the_others():
    # f0 has 4 chunks, f1 40, equal weights: after f0 is done f1 takes everything, and is on its fluid share throughout
    func, nbytes = _tickets([4000, 40000], [1, 1], 1000)
    worst, _ = bench.fluid_lag(func, nbytes, [1, 1], 1000, np.arange(len(func)))
    assert worst <= 1.0


def test_share_error_over_the_window_in_which_all_functions_are_active():
    func, nbytes = _tickets([300000, 300000, 300000], [1, 2, 3], 1000)
    t_end = np.cumsum(nbytes)            # uniform byte rate
    span, err, tenths, ntick = bench._share_errors(0, t_end, func, nbytes, np.array([1.0, 2.0, 3.0]))
    # the window ends when the weight-3 function is done: it holds 100 rounds of the order
    assert ntick == 600 and span == 600000
    assert err < 0.01 and all(t is not None and t < 0.05 for t in tenths)
    # shares swapped between two functions show up as an error of the size of the swap
    wrong = func.copy()
    wrong[func == 0], wrong[func == 1] = 1, 0
    _, err_wrong, _, _ = bench._share_errors(0, t_end, wrong, nbytes, np.array([1.0, 2.0, 3.0]))
    assert err_wrong > 0.4


def test_busy_time_is_the_union_of_the_launch_intervals():
    assert bench.busy_ms([]) == 0.0
    assert bench.busy_ms([(0.0, 1.0), (2.0, 3.0)]) == 2.0
    assert bench.busy_ms([(0.0, 2.0), (1.0, 3.0)]) == 3.0
    assert bench.busy_ms([(1.0, 3.0), (0.0, 4.0), (3.5, 3.6)]) == 4.0
