"""Pins for oracle/straggler_oracle.py (Sec. 3.1 of the paper).  None of them
re-types the oracle's expressions: order statistics are checked against their
counting definition, against the message-queue replay of Algorithm 4 and
against closed forms; the interpolation against the two iteration counts the
paper prints; the product table against a hand-worked case and exact
rationals."""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import workloads as wl
from oracle import brute
from oracle import bsgd_oracle as orc
from oracle import straggler_oracle as so

GOLD = os.path.join(os.path.dirname(__file__), "golden", "iterations_to_converge.json")


def _paper_points():
    with open(GOLD) as f:
        return [tuple(p) for p in json.load(f)["measured"]]


# ---------------------------------------------------------------------------
# time to collect k gradients
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(5))
def test_kth_time_counting_definition(seed):
    r = np.random.default_rng(seed)
    a = r.exponential(1.0, (7, 13)).astype(np.float32)
    a[2, 3] = a[2, 4]                                       # a tie
    kth = so.kth_arrival_times(a)
    assert kth.shape == a.shape and kth.dtype == np.float32
    for i in range(a.shape[0]):
        for k in range(1, a.shape[1] + 1):
            t = kth[i, k - 1]
            assert np.sum(a[i] <= t) >= k                   # by then k gradients are in
            assert np.sum(a[i] < t) <= k - 1                # and a moment earlier they were not


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_kth_time_is_the_wait_of_the_collect_loop(name):
    # Algorithm 4 with N = k stops at the k-th arrival: replay it, and ask the selection oracle too
    cfg = wl.get_config(name)
    a = wl.arrival_matrix(cfg, 6)
    kth = so.kth_arrival_times(a)
    for i in range(a.shape[0]):
        for k in (1, 2, cfg.N, cfg.W):
            kept = brute.ps_collect(a[i], k)
            assert a[i][kept[-1]] == kth[i, k - 1]
            sel, t_step = orc.select_first_n(a[i], k, cfg.W - k)
            assert np.float32(t_step) == kth[i, k - 1]


def test_never_arriving_gradients_come_last_as_inf():
    a = np.array([[3.0, np.inf, 1.0, np.nan, 2.0]], np.float32)
    kth = so.kth_arrival_times(a)
    assert kth[0, :3].tolist() == [1.0, 2.0, 3.0] and np.all(np.isinf(kth[0, 3:]))
    m = so.mean_kth_time(np.vstack([a, [[1, 2, 3, 4, 5]]]).astype(np.float32))
    assert m[:3].tolist() == [1.0, 2.0, 3.0] and np.all(np.isinf(m[3:]))


def test_single_vector_is_one_iteration():
    assert so.kth_arrival_times(np.array([2.0, 1.0], np.float32)).tolist() == [[1.0, 2.0]]


def test_mean_kth_exponential_closed_form():
    # k-th of W unit exponentials: E = sum_{i=0}^{k-1} 1/(W-i), Var = sum 1/(W-i)^2
    B, W = 40000, 12
    a = np.random.default_rng(3).exponential(1.0, (B, W)).astype(np.float32)
    m = so.mean_kth_time(a)
    for k in range(1, W + 1):
        mean = sum(1.0 / (W - i) for i in range(k))
        sd = math.sqrt(sum(1.0 / (W - i) ** 2 for i in range(k)) / B)
        assert abs(m[k - 1] - mean) < 5 * sd, (k, m[k - 1], mean)


def test_mean_kth_uniform_closed_form():
    B, W = 40000, 9
    a = np.random.default_rng(4).random((B, W)).astype(np.float32)
    m = so.mean_kth_time(a)
    for k in range(1, W + 1):
        p = k / (W + 1)
        sd = math.sqrt(p * (1 - p) / (W + 2) / B)
        assert abs(m[k - 1] - p) < 5 * sd


def test_mean_kth_exact_small():
    a = np.array([[0.5, 0.25, 4.0], [1.0, 8.0, 2.0], [3.0, 3.0, 0.125]], np.float32)
    want = [Fraction(0.25) + 1 + Fraction(0.125), Fraction(0.5) + 2 + 3, Fraction(4) + 8 + 3]
    got = so.mean_kth_time(a)
    assert [Fraction(float(x)) for x in got * 3] == want    # dyadic values: exact in fp64


# ---------------------------------------------------------------------------
# iterations to converge: the measured points and straight lines between them
# ---------------------------------------------------------------------------
def test_iterations_reproduce_the_printed_points_and_their_midpoint():
    pts = _paper_points()
    assert so.iterations_to_converge(50, pts) == 137.5e3
    assert so.iterations_to_converge(100, pts) == 76.2e3
    assert so.iterations_to_converge(75, pts) == pytest.approx((137.5e3 + 76.2e3) / 2, rel=1e-15)
    # "nearly halves" when N doubles
    assert 0.5 < so.iterations_to_converge(100, pts) / so.iterations_to_converge(50, pts) < 0.6


def test_iterations_outside_the_measured_range_are_unknown():
    pts = _paper_points()
    assert math.isnan(so.iterations_to_converge(49, pts))
    assert math.isnan(so.iterations_to_converge(101, pts))
    assert math.isnan(so.iterations_to_converge(5, []))


def test_iterations_piecewise_linear_against_numpy_interp():
    pts = [(50, 137.5e3), (70, 101e3), (80, 93e3), (90, 84e3), (100, 76.2e3)]
    shuffled = [pts[i] for i in (3, 0, 4, 2, 1)]              # order of the table does not matter
    xs, ys = zip(*pts)
    for N in range(50, 101):
        assert so.iterations_to_converge(N, shuffled) == pytest.approx(float(np.interp(N, xs, ys)), rel=1e-14)


# ---------------------------------------------------------------------------
# estimated time to converge and the best split
# ---------------------------------------------------------------------------
def test_time_to_converge_hand_worked():
    # 4 machines; measured: N=2 -> 100 iterations, N=4 -> 50 (so N=3 -> 75)
    est, best = so.time_to_converge([1.0, 2.0, 3.0, 10.0], [(2, 100), (4, 50)])
    assert math.isnan(est[0]) and est[1:].tolist() == [200.0, 225.0, 500.0]
    assert best == 2
    # without the straggling last gradient more workers win
    est, best = so.time_to_converge([1.0, 2.0, 2.1, 2.2], [(2, 100), (4, 50)])
    assert est[1:].tolist() == pytest.approx([200.0, 157.5, 110.0]) and best == 4


def test_time_to_converge_ties_go_to_more_workers_and_unknown_is_never_chosen():
    est, best = so.time_to_converge([1.0, 1.0, 2.0, 4.0], [(2, 8), (4, 2)])      # 8, 10, 8
    assert est[1:].tolist() == [8.0, 10.0, 8.0] and best == 4
    est, best = so.time_to_converge([1.0, 1.0], [(5, 10), (6, 9)])
    assert np.all(np.isnan(est)) and best == 0
    est, best = so.time_to_converge([1.0, np.inf], [(1, 10), (2, 5)])            # the last gradient never comes
    assert best == 1


@pytest.mark.parametrize("seed", range(4))
def test_time_to_converge_exact_replay(seed):
    r = np.random.default_rng(seed)
    W = 12
    mean = np.sort(r.integers(1, 2000, W) / 64.0)                                # dyadic: exact products
    pts = [(4, 4096), (8, 1024), (12, 512)]
    est, best = so.time_to_converge(mean, pts)
    want = {}
    for N in range(4, 13):
        (n0, i0), (n1, i1) = [(p, q) for p, q in zip(pts[:-1], pts[1:]) if p[0] <= N <= q[0]][0]
        it = Fraction(i0) + Fraction(N - n0, n1 - n0) * (i1 - i0)
        want[N] = it * Fraction(float(mean[N - 1]))
    for N, w in want.items():
        assert Fraction(float(est[N - 1])) == w
    lo = min(want.values())
    assert best == max(N for N, w in want.items() if w == lo)


def test_paper_shaped_pool_prefers_a_few_backups():
    # 100 machines with a long-tailed arrival distribution (Sec. 3.1): waiting for
    # everybody is not the fastest split, and neither is dropping half of them
    cfg = wl.get_config("C2")
    a = wl.arrival_matrix(cfg, 4000, workers=100)
    est, best = so.time_to_converge(so.mean_kth_time(a), _paper_points())
    assert 80 <= best < 100, best
    assert est[best - 1] < est[99] and est[best - 1] < est[49]
